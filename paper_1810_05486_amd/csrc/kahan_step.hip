// Fused lazy-update kernel (Algorithm 1 of the paper, Section 2): one launch
// walks every tile of every tensor of a list.
//
// Work distribution: a persistent grid of wavefronts; wave w takes tiles
// w, w + W, w + 2W, ... of the tile table, so at any moment the grid streams
// one contiguous window of the parameter set.  A tile is 4096 elements of one
// tensor; a lane handles 16 consecutive elements per pass (one dwordx4 of int8
// theta, one of comp, two of int16 grad), four passes per tile with all loads
// issued before the arithmetic.
//
// Arithmetic: two paths with identical results.
//   * generic: 64-bit integers, any widths / shifts / grid move / decay /
//     no-accumulator mode inside the documented domain;
//   * fast: 32-bit, chosen per tensor when the shifts allow it.  The step
//     RNE(-lr*g / 2^k) is ONE fp32 fused multiply-add: g and lr are exact in
//     fp32, the FMA forms their product exactly and adds 1.5*2^(23+k), whose
//     ulp is 2^k, so the single IEEE rounding of the FMA *is* the
//     round-to-nearest-even at bit k and the integer falls out of the
//     significand bits.  The decay term uses the same construction in fp64.
//
// Running maximum of |v| per tensor: per-lane max, DPP wave reduction when a
// wave moves to another tensor, LDS stage across the four waves of a block at
// the end, one atomic per (block, tensor).
#include "step_common.hpp"

namespace lpk {

struct StepParams {
  int      path;            // 0 skip, 1 generic, 2 fast
  int      wt, wc, wg, d;
  int      has_comp;
  int      kg;              // shift of the gradient term: fl_g + 16 - F
  int      kw;              // shift of the decay term: 32 - d
  int      u, kth, kc;      // grid move: v_G = v << u; theta' = RNE(v_G >> kth); c' = RNE(r >> kc)
  int64_t  lr, lrwd;
  int      qmin_t, qmax_t, qmin_c, qmax_c;
  // fast path constants
  float    nlr_f;  float magic_f;  int magic_fi;
  double   nlrwd_d; double magic_d; int magic_dlo;
  int      half_m1;         // 2^(d-1) - 1
};

// ---------------------------------------------------------------- generic (int64)


__device__ __forceinline__ void update_generic(const StepParams& p, int64_t th, int64_t c, int64_t g,
                                               int& th_new, int& c_new, uint64_t& vabs)
{
  int64_t s = rescale_cap64(-p.lr * g, p.kg);
  if (p.lrwd) s += rescale_cap64(-p.lrwd * th, p.kw);
  int64_t v = th * (1ll << p.d) + c + s;
  vabs = (uint64_t)(v < 0 ? -v : v);
  int64_t vG = v * (1ll << p.u);
  int64_t tn = rne_shr64(vG, p.kth);
  tn = tn > p.qmax_t ? p.qmax_t : (tn < p.qmin_t ? p.qmin_t : tn);
  int64_t r  = vG - tn * (1ll << p.kth);
  int64_t cn = rne_shr64(r, p.kc);
  cn = cn > p.qmax_c ? p.qmax_c : (cn < p.qmin_c ? p.qmin_c : cn);
  th_new = (int)tn; c_new = (int)cn;
}


// Element-at-a-time tile: any alignment, any widths.  Lane l takes elements l, l+64, ...
__device__ __forceinline__ uint64_t tile_generic(const StepParams& p, const TensorDev& T, uint64_t off, uint32_t cnt, int lane)
{
  uint64_t vm = 0;
  for (uint32_t j = lane; j < cnt; j += kWave) {
    uint64_t i = off + j;
    int th = load_elem(T.theta, i, p.wt);
    int c  = p.has_comp ? load_elem(T.comp, i, p.wc) : 0;
    int g  = load_elem(T.grad, i, p.wg);
    int tn, cn; uint64_t va;
    update_generic(p, th, c, g, tn, cn, va);
    vm = va > vm ? va : vm;
    store_elem(T.theta, i, p.wt, tn);
    if (p.has_comp) store_elem(T.comp, i, p.wc, cn);
  }
  return vm;
}

// ---------------------------------------------------------------- fast (int32 + FMA rounding)

template <bool DECAY>
__device__ __forceinline__ void update_fast(const StepParams& p, int th, int c, int g, int& tn, int& cn, int& vmx, int& vmn)
{
#ifdef LPK_NO_MATH
  tn = th ^ (g & 1); cn = c; vmx = max(vmx, g); return;
#endif
  int s = __float_as_int(__builtin_fmaf((float)g, p.nlr_f, p.magic_f)) - p.magic_fi;
  if (DECAY) {
    double r = __builtin_fma((double)th, p.nlrwd_d, p.magic_d);
    s += __double2loint(r) - p.magic_dlo;
  }
  int v = (th << p.d) + c + s;          // th << d on a negative th: two's complement, what the hardware does
  vmx = v > vmx ? v : vmx;
  vmn = v < vmn ? v : vmn;
  int q = (v + p.half_m1 + ((v >> p.d) & 1)) >> p.d;      // RNE(v / 2^d), d >= 1, no overflow by path choice
  tn = min(max(q, p.qmin_t), p.qmax_t);
  int r = v - (tn << p.d);
  cn = min(max(r, p.qmin_c), p.qmax_c);
}


// 16 consecutive elements per lane; W = width of theta and comp (8 or 16), grads int16.
template <int W> struct Group;
template <> struct Group<8>  { v4i th;      v4i c;      v4i g[2]; };
template <> struct Group<16> { v4i th[2];   v4i c[2];   v4i g[2]; };

__device__ __forceinline__ void load_group(Group<8>& G, const TensorDev& T, uint64_t e)
{
  G.th   = ld_stream((const v4i*)((const int8_t*)T.theta + e));
  G.c    = ld_stream((const v4i*)((const int8_t*)T.comp + e));
  G.g[0] = ld_stream((const v4i*)((const int16_t*)T.grad + e));
  G.g[1] = ld_stream((const v4i*)((const int16_t*)T.grad + e + 8));
}
__device__ __forceinline__ void load_group(Group<16>& G, const TensorDev& T, uint64_t e)
{
  G.th[0] = ld_stream((const v4i*)((const int16_t*)T.theta + e));
  G.th[1] = ld_stream((const v4i*)((const int16_t*)T.theta + e + 8));
  G.c[0]  = ld_stream((const v4i*)((const int16_t*)T.comp + e));
  G.c[1]  = ld_stream((const v4i*)((const int16_t*)T.comp + e + 8));
  G.g[0]  = ld_stream((const v4i*)((const int16_t*)T.grad + e));
  G.g[1]  = ld_stream((const v4i*)((const int16_t*)T.grad + e + 8));
}


template <bool DECAY>
__device__ __forceinline__ void compute_store_group(const StepParams& p, Group<8>& G, const TensorDev& T, uint64_t e, int& vmx, int& vmn)
{
  v4i to, co;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    int tn[4], cn[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      int k = w * 4 + b;                     // element within the group
      update_fast<DECAY>(p, sx8(G.th[w], b), sx8(G.c[w], b), sx16(G.g[k >> 3][(k >> 1) & 3], k & 1), tn[b], cn[b], vmx, vmn);
    }
    to[w] = pack4x8(tn[0], tn[1], tn[2], tn[3]);
    co[w] = pack4x8(cn[0], cn[1], cn[2], cn[3]);
  }
  st_stream((v4i*)((int8_t*)T.theta + e), to);
  st_stream((v4i*)((int8_t*)T.comp + e), co);
}

template <bool DECAY>
__device__ __forceinline__ void compute_store_group(const StepParams& p, Group<16>& G, const TensorDev& T, uint64_t e, int& vmx, int& vmn)
{
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    v4i to, co;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      int tn[2], cn[2];
#pragma unroll
      for (int h = 0; h < 2; ++h)
        update_fast<DECAY>(p, sx16(G.th[q][w], h), sx16(G.c[q][w], h), sx16(G.g[q][w], h), tn[h], cn[h], vmx, vmn);
      to[w] = pack2x16(tn[0], tn[1]);
      co[w] = pack2x16(cn[0], cn[1]);
    }
    st_stream((v4i*)((int16_t*)T.theta + e + 8 * q), to);
    st_stream((v4i*)((int16_t*)T.comp + e + 8 * q), co);
  }
}

// Vector tile: full 16-element groups with the fast arithmetic, the ragged end element by element.
template <int W, bool DECAY>
__device__ __forceinline__ uint64_t tile_fast(const StepParams& p, const TensorDev& T, uint64_t off, uint32_t cnt, int lane)
{
  int vmx = 0, vmn = 0;
  const uint32_t ngroups = cnt / kGroup;
  if (ngroups == kWave * kPasses) {                       // full tile: every load issued before any arithmetic
    Group<W> G[kPasses];
#pragma unroll
    for (int ps = 0; ps < kPasses; ++ps) load_group(G[ps], T, off + (uint64_t)(ps * kWave + lane) * kGroup);
#pragma unroll
    for (int ps = 0; ps < kPasses; ++ps)
      compute_store_group<DECAY>(p, G[ps], T, off + (uint64_t)(ps * kWave + lane) * kGroup, vmx, vmn);
  } else {
    for (uint32_t gi = lane; gi < ngroups; gi += kWave) {
      Group<W> G;
      uint64_t e = off + (uint64_t)gi * kGroup;
      load_group(G, T, e);
      compute_store_group<DECAY>(p, G, T, e, vmx, vmn);
    }
  }
  int64_t a = vmx, b = -(int64_t)vmn;
  uint64_t vm = (uint64_t)(a > b ? a : b);
  const uint32_t tail = cnt - ngroups * kGroup;           // < 16 elements
  if (tail) {
    uint64_t t2 = tile_generic(p, T, off + (uint64_t)ngroups * kGroup, tail, lane);
    vm = t2 > vm ? t2 : vm;
  }
  return vm;
}

// One pipeline stage: start the loads of the wave's next tile into `nxt` if that tile continues the run
// (same tensor, full), then compute and store `cur`.  Returns whether `nxt` was filled; ti/off advance to it.
template <bool DECAY>
__device__ __forceinline__ bool stage_fast8(const StepParams& p, const TensorDev& T, const Tile* __restrict__ tiles,
                                            uint32_t n_tiles, uint32_t nw, uint32_t& ti, uint64_t& off, int tensor, int lane,
                                            Group<8> (&cur)[kPasses], Group<8> (&nxt)[kPasses], int& vmx, int& vmn)
{
  const uint32_t tn = ti + nw;
  bool more = false;
  uint64_t noff = 0;
  if (tn < n_tiles) {
    const Tile nx = tiles[tn];
    more = wave_uniform((int)nx.tensor) == tensor && (uint32_t)wave_uniform((int)nx.count) == (uint32_t)kTileElems;
    noff = ((uint64_t)(uint32_t)wave_uniform((int)(nx.offset >> 32)) << 32) | (uint32_t)wave_uniform((int)nx.offset);
  }
  if (more) {
#pragma unroll
    for (int ps = 0; ps < kPasses; ++ps) load_group(nxt[ps], T, noff + (uint64_t)(ps * kWave + lane) * kGroup);
  }
#pragma unroll
  for (int ps = 0; ps < kPasses; ++ps)
    compute_store_group<DECAY>(p, cur[ps], T, off + (uint64_t)(ps * kWave + lane) * kGroup, vmx, vmn);
  if (more) { ti = tn; off = noff; }
  return more;
}

// Processes the full tile at (ti, off) and every following tile of this wave that continues the run; on
// return ti is the last tile consumed (the caller's loop increment moves past it).
template <bool DECAY>
__device__ __forceinline__ uint64_t run_fast8(const StepParams& p, const TensorDev& T, const Tile* __restrict__ tiles,
                                              uint32_t n_tiles, uint32_t nw, uint32_t& ti, uint64_t off, int tensor, int lane)
{
  int vmx = 0, vmn = 0;
  Group<8> A[kPasses], B[kPasses];
#pragma unroll
  for (int ps = 0; ps < kPasses; ++ps) load_group(A[ps], T, off + (uint64_t)(ps * kWave + lane) * kGroup);
  while (true) {
    if (!stage_fast8<DECAY>(p, T, tiles, n_tiles, nw, ti, off, tensor, lane, A, B, vmx, vmn)) break;
    if (!stage_fast8<DECAY>(p, T, tiles, n_tiles, nw, ti, off, tensor, lane, B, A, vmx, vmn)) break;
  }
  int64_t a = vmx, b = -(int64_t)vmn;
  return (uint64_t)(a > b ? a : b);
}

// ---------------------------------------------------------------- per-tensor set-up (wave-uniform)

__device__ __forceinline__ void setup_tensor(StepParams& p, const TensorDev& T, int fl_in, int fl_out, int fl_g,
                                             uint32_t lr, uint32_t wd, uint32_t& status_bits)
{
  p.wt = T.wt; p.wc = T.wc; p.wg = T.wg; p.has_comp = T.comp != nullptr;
  p.d = p.has_comp ? T.d : 0;
  const int delta = fl_out - fl_in;
  if (fl_in < kFlMin || fl_in > kFlMax || fl_out < kFlMin || fl_out > kFlMax || fl_g < kFlMin || fl_g > kFlMax ||
      p.d > kDMax || delta > kDeltaMax || delta < -kDeltaMax) {
    p.path = 0; status_bits |= kStatusDomain; return;
  }
  const int F = fl_in + p.d;
  p.kg = fl_g + 16 - F;
  p.kw = 32 - p.d;
  p.u = delta > 0 ? delta : 0;
  p.kth = p.d + p.u - delta;
  p.kc = p.kth - p.d;
  p.lr = lr; p.lrwd = (int64_t)lr * (int64_t)wd;
  p.qmax_t = (1 << (p.wt - 1)) - 1; p.qmin_t = -(1 << (p.wt - 1));
  const int wc = p.has_comp ? p.wc : 8;
  p.qmax_c = (1 << (wc - 1)) - 1;   p.qmin_c = -(1 << (wc - 1));
  p.path = 1;

  // Fast path: same-width theta/comp with int16 grads on 16-byte aligned buffers, no grid move,
  // 1 <= d, a step shift k with |lr * g| <= lr * 2^15 < 2^(22+k) (so the fp32 FMA rounding trick is exact
  // and |s| < 2^22), and every intermediate provably inside int32.
  if (!p.has_comp || !T.vec_step || p.wt != p.wc || p.wg != 16 || delta != 0 || p.d < 1 || p.kg < 1) return;
  if (p.kg < 9 && ((int64_t)lr << 15) >= (1ll << (22 + p.kg))) return;
  int64_t bound = (1ll << (p.wt - 1 + p.d)) + (1ll << (p.wc - 1));             // |theta * 2^d| + |c|
  bound += p.kg < 40 ? (((int64_t)lr << 15) >> p.kg) + 1 : 0;                   // |s_g|
  int64_t sw = 0;
  if (p.lrwd) sw = ((p.lrwd << (p.wt - 1)) >> p.kw) + 1;                        // |s_w|
  bound += sw;
  bound += 1ll << (p.d - 1);                                                    // the rounding addend
  if (bound >= (1ll << 31)) return;
  p.path = 2;
  const int kg = p.kg > 40 ? 40 : p.kg;                                         // k >= 32 already gives s = 0
  p.magic_fi = ((127 + 23 + kg) << 23) | 0x400000;                              // 1.5 * 2^(23 + k)
  p.magic_f  = __int_as_float(p.magic_fi);
  p.nlr_f    = -(float)lr;
  const long long md = ((long long)(1023 + 52 + p.kw) << 52) | (1ll << 51);     // 1.5 * 2^(52 + kw)
  p.magic_d   = __longlong_as_double(md);
  p.magic_dlo = (int)(md & 0xffffffffll);
  p.nlrwd_d   = -(double)p.lrwd;
  p.half_m1   = (1 << (p.d - 1)) - 1;
}

// ---------------------------------------------------------------- the kernel


__global__ void __launch_bounds__(kBlock)
kahan_step_kernel(const TensorDev* __restrict__ tensors, const Tile* __restrict__ tiles, uint32_t n_tiles,
                  const int32_t* __restrict__ fl_in, const int32_t* __restrict__ fl_out, const int32_t* __restrict__ fl_g,
                  uint32_t lr, uint32_t wd, uint64_t* vmax, uint32_t* status)
{
  __shared__ int      s_tensor[kWavesPerBlock];
  __shared__ uint64_t s_max[kWavesPerBlock];

  const int lane   = threadIdx.x & (kWave - 1);
  const int wave   = wave_uniform(threadIdx.x >> 6);
  const uint32_t w0 = blockIdx.x * kWavesPerBlock + wave;
  const uint32_t nw = gridDim.x * kWavesPerBlock;

  int cur = -1;
  uint64_t lane_max = 0;
  uint32_t status_bits = 0;
  StepParams p; p.path = 0;
  TensorDev T;

  for (uint32_t ti = w0; ti < n_tiles; ti += nw) {      // ti may also be advanced inside by a pipelined run
    const Tile tl = tiles[ti];
    const int t = wave_uniform((int)tl.tensor);
    const uint32_t cnt = (uint32_t)wave_uniform((int)tl.count);
    const uint64_t off = ((uint64_t)(uint32_t)wave_uniform((int)(tl.offset >> 32)) << 32) | (uint32_t)wave_uniform((int)tl.offset);
    if (t != cur) {
      if (cur >= 0 && vmax) flush_wave(vmax, cur, lane_max, lane);
      lane_max = 0;
      cur = t;
      T = tensors[t];
      setup_tensor(p, T, fl_in[t], fl_out[t], fl_g[t], lr, wd, status_bits);
    }
    uint64_t vm = 0;
    if (p.path == 2) {
      if (p.wt == 8 && cnt == (uint32_t)kTileElems) {
        // Run of full int8 tiles of this tensor, software-pipelined: the loads of the wave's next tile are in
        // flight while the current one is computed and stored, so the memory pipe never waits for the ALU.
        vm = p.lrwd ? run_fast8<true>(p, T, tiles, n_tiles, nw, ti, off, cur, lane)
                    : run_fast8<false>(p, T, tiles, n_tiles, nw, ti, off, cur, lane);
      }
      else if (p.wt == 8) vm = p.lrwd ? tile_fast<8, true>(p, T, off, cnt, lane)  : tile_fast<8, false>(p, T, off, cnt, lane);
      else                vm = p.lrwd ? tile_fast<16, true>(p, T, off, cnt, lane) : tile_fast<16, false>(p, T, off, cnt, lane);
    } else if (p.path == 1) {
      vm = tile_generic(p, T, off, cnt, lane);
    }
    lane_max = vm > lane_max ? vm : lane_max;
  }

  if (status && status_bits && lane == 0) atomicOr(status, status_bits);

  // LDS stage: the four waves of a block usually end on the same tensor.
  if (vmax) flush_block(vmax, cur, lane_max, lane, wave, s_tensor, s_max);
}

__global__ void __launch_bounds__(kBlock) fill_u64_kernel(uint64_t* p, uint32_t n, uint64_t v)
{
  uint32_t i = blockIdx.x * kBlock + threadIdx.x;
  if (i < n) p[i] = v;
}

hipError_t launch_kahan_step(const TensorDev* tensors, const Tile* tiles, uint32_t n_tiles, uint32_t n_tensors, uint32_t grid,
                             const int32_t* fl_in, const int32_t* fl_out, const int32_t* fl_g, uint32_t lr, uint32_t wd,
                             uint64_t* vmax, uint32_t* status, hipStream_t stream)
{
  if (vmax) {
    hipLaunchKernelGGL(fill_u64_kernel, dim3((n_tensors + kBlock - 1) / kBlock), dim3(kBlock), 0, stream, vmax, n_tensors, 0ull);
  }
  if (n_tiles) {
    hipLaunchKernelGGL(kahan_step_kernel, dim3(grid), dim3(kBlock), 0, stream, tensors, tiles, n_tiles,
                       fl_in, fl_out, fl_g, lr, wd, vmax, status);
  }
  return hipGetLastError();
}

}  // namespace lpk

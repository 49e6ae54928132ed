// Pieces shared by the update kernels (plain lazy update, momentum, ADAM): the persistent walk over the tile table,
// the groups-in-flight loop of a tile, the last stage of Algorithm 1 (compensated sum -> new parameter and new
// accumulator) in its three arithmetic forms, exact fp64 helpers, element and vector accesses, byte/halfword
// unpacking, the per-tensor maxima flush, stores that skip unchanged data.
#pragma once
#include "lpk_device.hpp"

namespace lpk {

// Exact fp64 helpers of the wide arithmetic: 2^k for -1022 <= k <= 1023, and a clamp.
__device__ __forceinline__ double pow2d(int k) { return __longlong_as_double((long long)(1023 + k) << 52); }
__device__ __forceinline__ double clampd(double x, double lo, double hi) { return __builtin_fmin(__builtin_fmax(x, lo), hi); }

// Median of three (a clamp when lo <= hi) and the 24-bit multiply-add, as single VALU operations.
__device__ __forceinline__ int med3_i32(int x, int lo, int hi)
{
  int r;
  asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "v"(lo), "v"(hi));
  return r;
}

__device__ __forceinline__ int mad_i24(int a, int b, int c)          // sext24(a) * sext24(b) + c
{
  int r;
  asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

__device__ __forceinline__ int load_elem(const void* p, uint64_t i, int bits)
{
  return bits == 8 ? (int)((const int8_t*)p)[i] : (int)((const int16_t*)p)[i];
}
__device__ __forceinline__ void store_elem(void* p, uint64_t i, int bits, int v)
{
  if (bits == 8) ((int8_t*)p)[i] = (int8_t)v; else ((int16_t*)p)[i] = (int16_t)v;
}

// Streaming accesses: global address space (global_load/global_store, not flat), non-temporal.
template <typename V> __device__ __forceinline__ V ld_stream(const V* p)
{
#if LPK_NT_LOAD
  return __builtin_nontemporal_load((const LPK_GLOBAL V*)p);
#else
  return *(const LPK_GLOBAL V*)p;
#endif
}
template <typename V> __device__ __forceinline__ void st_stream(V* p, V v)
{
#if LPK_NT_STORE
  __builtin_nontemporal_store(v, (LPK_GLOBAL V*)p);
#else
  *(LPK_GLOBAL V*)p = v;
#endif
}

typedef int v4i __attribute__((ext_vector_type(4)));

// Where an update kernel takes its gradients from: the int16 array, the fp32 source quantized in registers, or an
// int8 array (the all-8-bit mode of Section 4; vector path of the plain update with 8-bit theta and comp).
enum { kGradI16 = 0, kGradF32 = 1, kGradI8 = 2 };

// One fp32 gradient onto the int16 grid exactly as the quantization kernel does it: x * 2^fl is exact in fp32,
// v_rndne rounds half to even, the rails clamp, NaN becomes 0.  The result is an integer-valued float.  `ab_max`
// collects the largest |bit pattern| seen (>= 0x7f800000 means a NaN or Inf went by).
__device__ __forceinline__ float quant_f32(float x, float scale, float lo, float hi, uint32_t& ab_max)
{
  const uint32_t ab = __float_as_uint(x) & 0x7fffffffu;
  ab_max = ab > ab_max ? ab : ab_max;
  float y = __builtin_rintf(x * scale);
  y = __builtin_fminf(__builtin_fmaxf(y, lo), hi);
  return ab > 0x7f800000u ? 0.0f : y;
}

// A tensor that a kernel fed from the fp32 gradients skips for its domain (path -1 in the kernels' parameter blocks:
// some fraclen other than the gradients' is out of range): the quantization the call stands for would still have
// looked at the gradients and reported a NaN or an infinity among them, so the status word must too.
constexpr int kPathSkipButScan = -1;
__device__ __forceinline__ void scan_nonfinite(const void* src, uint64_t off, uint32_t cnt, int lane, uint32_t& ab_max)
{
  const uint32_t* s = (const uint32_t*)src + off;
  for (uint32_t j = lane; j < cnt; j += kWave) {
    const uint32_t ab = s[j] & 0x7fffffffu;
    ab_max = ab > ab_max ? ab : ab_max;
  }
}
template <int GS> __device__ __forceinline__ int skipped_path(int fl_g)
{
  return GS == kGradF32 && fl_g >= kFlMin && fl_g <= kFlMax ? kPathSkipButScan : 0;
}

__device__ __forceinline__ int sx8(int w, int b)  { return (int)(int8_t)(w >> (8 * b)); }
__device__ __forceinline__ int sx16(int w, int h) { return (int)(int16_t)(w >> (16 * h)); }

__device__ __forceinline__ void flush_wave(uint64_t* vmax, int tensor, uint64_t lane_max, int lane)
{
  uint64_t m = wave_max_u64(lane_max);
  if (lane == 0 && m) atomicMax((unsigned long long*)&vmax[tensor], (unsigned long long)m);
}

// Low bytes of four ints -> one dword (a in byte 0), low halves of two ints -> one dword (a low), via
// v_perm_b32: selector bytes 0-3 pick bytes of the second operand, 4-7 of the first, 0x0c gives 0x00.
__device__ __forceinline__ int pack4x8(int a, int b, int c, int d)
{
  const uint32_t lo = __builtin_amdgcn_perm((uint32_t)b, (uint32_t)a, 0x0c0c0400u);
  const uint32_t hi = __builtin_amdgcn_perm((uint32_t)d, (uint32_t)c, 0x0c0c0400u);
  return (int)(lo | (hi << 16));
}
__device__ __forceinline__ int pack2x16(int a, int b)
{
  return (int)__builtin_amdgcn_perm((uint32_t)b, (uint32_t)a, 0x05040100u);
}

// 16 consecutive W-bit elements of one lane: load (one or two dwordx4), pick the k-th, pack and store.
template <int W> __device__ __forceinline__ void load16(v4i (&dst)[W / 8], const void* base, uint64_t e)
{
  if (W == 8) dst[0] = ld_stream((const v4i*)((const int8_t*)base + e));
  else { dst[0] = ld_stream((const v4i*)((const int16_t*)base + e)); dst[W / 8 - 1] = ld_stream((const v4i*)((const int16_t*)base + e + 8)); }
}
template <int W> __device__ __forceinline__ int elem16(const v4i (&src)[W / 8], int k)        // k-th of 16 elements
{
  if (W == 8) return sx8(src[0][k >> 2], k & 3);
  return sx16(src[(W / 8 - 1) * (k >> 3)][(k >> 1) & 3], k & 1);
}
template <int W> __device__ __forceinline__ void store16(void* base, uint64_t e, const int (&val)[16])
{
  if (W == 8) {
    v4i o;
#pragma unroll
    for (int w = 0; w < 4; ++w) o[w] = pack4x8(val[4 * w], val[4 * w + 1], val[4 * w + 2], val[4 * w + 3]);
    st_stream((v4i*)((int8_t*)base + e), o);
  } else {
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      v4i o;
#pragma unroll
      for (int w = 0; w < 4; ++w) o[w] = pack2x16(val[8 * q + 2 * w], val[8 * q + 2 * w + 1]);
      st_stream((v4i*)((int16_t*)base + e + 8 * q), o);
    }
  }
}

// E consecutive elements of one lane as 1, 2 or 4 dwords per array: load, pick the k-th element, pack, store.
typedef int v2i __attribute__((ext_vector_type(2)));
template <int N> struct DW { int d[N]; };                 // N = 1, 2 or 4 dwords moved by one access

template <int N> __device__ __forceinline__ DW<N> ld_dw(const void* p)
{
  DW<N> r;
  if constexpr (N == 1) { r.d[0] = ld_stream((const int*)p); }
  else if constexpr (N == 2) { v2i v = ld_stream((const v2i*)p); r.d[0] = v[0]; r.d[1] = v[1]; }
  else { v4i v = ld_stream((const v4i*)p); r.d[0] = v[0]; r.d[1] = v[1]; r.d[2] = v[2]; r.d[3] = v[3]; }
  return r;
}
template <int N> __device__ __forceinline__ void st_dw(void* p, const DW<N>& r)
{
  if constexpr (N == 1) { st_stream((int*)p, r.d[0]); }
  else if constexpr (N == 2) { v2i v; v[0] = r.d[0]; v[1] = r.d[1]; st_stream((v2i*)p, v); }
  else { v4i v; v[0] = r.d[0]; v[1] = r.d[1]; v[2] = r.d[2]; v[3] = r.d[3]; st_stream((v4i*)p, v); }
}
template <int W, int N> __device__ __forceinline__ int elem_dw(const DW<N>& r, int k)
{
  if constexpr (W == 8) return sx8(r.d[k >> 2], k & 3); else return sx16(r.d[k >> 1], k & 1);
}
template <int W, int E> __device__ __forceinline__ DW<E * W / 32> pack_dw(const int (&val)[E])
{
  DW<E * W / 32> r;
#pragma unroll
  for (int w = 0; w < E * W / 32; ++w) {
    if constexpr (W == 8) r.d[w] = pack4x8(val[4 * w], val[4 * w + 1], val[4 * w + 2], val[4 * w + 3]);
    else                  r.d[w] = pack2x16(val[2 * w], val[2 * w + 1]);
  }
  return r;
}

// RNE(y / 2^b) for a wave-uniform 0 <= b <= 30 without a branch: `half_m1` = 2^(b-1) - 1 (0 when b == 0),
// `nz` = 1 when b > 0 else 0 (a zero-width bit-field extract yields 0, so b == 0 returns y itself).
// The caller has shown |y| + 2^(b-1) < 2^31.
__device__ __forceinline__ int rne_shr32(int y, int b, int half_m1, int nz)
{
  const int lsb = (int)__builtin_amdgcn_ubfe((uint32_t)y, (uint32_t)b, (uint32_t)nz);
  return (y + half_m1 + lsb) >> b;
}

// Block-level end of a persistent kernel: combine the four waves' (tensor, max) pairs in LDS, one atomic per tensor.
__device__ __forceinline__ void flush_block(uint64_t* vmax, int cur, uint64_t lane_max, int lane, int wave,
                                            int* s_tensor, uint64_t* s_max)
{
  uint64_t m = wave_max_u64(lane_max);
  if (lane == 0) { s_tensor[wave] = cur; s_max[wave] = m; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int a = 0; a < kWavesPerBlock; ++a) {
      int ta = s_tensor[a];
      if (ta < 0) continue;
      uint64_t ma = s_max[a];
      for (int b = a + 1; b < kWavesPerBlock; ++b)
        if (s_tensor[b] == ta) { ma = s_max[b] > ma ? s_max[b] : ma; s_tensor[b] = -1; }
      if (ma) atomicMax((unsigned long long*)&vmax[ta], (unsigned long long)ma);
    }
  }
  __syncthreads();
}

// ---------------------------------------------------------------- the walk over the tile table
//
// The callables handed to walk_tiles are lambdas that capture the kernel's state by reference; they must be
// inlined (LPK_INLINE_LAMBDA after the parameter list), or that state is forced out of registers into scratch
// memory.
#define LPK_INLINE_LAMBDA __attribute__((always_inline))
//
// A persistent grid of wavefronts: wave w takes tiles w, w + W, w + 2W, ... of the table, so at any moment the grid
// streams one contiguous window of the parameter set.  `leave(t)` runs when the walk moves on from tensor t (flush
// its maxima), `enter(t)` when it reaches a tile of another tensor (load its descriptor, derive its constants),
// `tile(off, cnt)` for every tile; all three are wave-uniform.  Returns the tensor the wave ended on, -1 if it
// had no tile.
template <typename Leave, typename Enter, typename TileFn>
__device__ __forceinline__ int walk_tiles(const Tile* __restrict__ tiles, uint32_t n_tiles, Leave&& leave, Enter&& enter, TileFn&& tile)
{
  const uint32_t w0 = blockIdx.x * kWavesPerBlock + (uint32_t)wave_uniform(threadIdx.x >> 6);
  const uint32_t nw = gridDim.x * kWavesPerBlock;
  int cur = -1;
  for (uint32_t ti = w0; ti < n_tiles; ti += nw) {
    int t; uint32_t cnt; uint64_t off;
    read_tile(tiles, ti, t, cnt, off);
    if (t != cur) {
      if (cur >= 0) leave(cur);
      cur = t;
      enter(t);
    }
    tile(off, cnt);
  }
  return cur;
}

// End of a persistent update kernel: raise the status bits a wave collected.
__device__ __forceinline__ void raise_status(uint32_t* status, uint32_t bits, int lane)
{
  if (status && bits && lane == 0) atomicOr(status, bits);
}

// ---------------------------------------------------------------- last stage of Algorithm 1
//
// v = theta * 2^d + c + s (the compensated sum on grid F) -> theta' = sat(RNE(v on theta's new grid)),
// c' = sat(RNE((v - theta') on the accumulator's new grid)), and the running maximum of |v|.  Three forms with
// identical results; which one a tensor takes is decided per tensor from its shifts (wave-uniform).

// wide: exact fp64, any shifts of the domain (grid moves included).  Every quantity is an integer below 2^53 times
// a power of two, so sums and power-of-two scalings are exact and v_rndne_f64 is the RNE of the definition.  The
// residual v_G - theta' * 2^kth is exact while it is below 2^53; beyond that the accumulator saturates whatever the
// last bits are.
struct Alg1Wide { double p2d, p2u, inv_kth, p2kth, inv_kc, lo_t, hi_t, lo_c, hi_c; };

__device__ __forceinline__ Alg1Wide make_alg1_wide(int d, int u, int kth, int kc, int qmin_t, int qmax_t, int qmin_c, int qmax_c)
{
  Alg1Wide a;
  a.p2d = pow2d(d); a.p2u = pow2d(u); a.inv_kth = pow2d(-kth); a.p2kth = pow2d(kth); a.inv_kc = pow2d(-kc);
  a.lo_t = (double)qmin_t; a.hi_t = (double)qmax_t; a.lo_c = (double)qmin_c; a.hi_c = (double)qmax_c;
  return a;
}

__device__ __forceinline__ void alg1_wide(const Alg1Wide& a, int th, int c, double s, int& tn, int& cn, double& vabs_max)
{
  const double v = __builtin_fma((double)th, a.p2d, (double)c) + s;
  vabs_max = __builtin_fmax(vabs_max, __builtin_fabs(v));
  const double vG = v * a.p2u;
  const double t = clampd(__builtin_rint(vG * a.inv_kth), a.lo_t, a.hi_t);
  const double rr = __builtin_fma(-t, a.p2kth, vG);
  const double cc = clampd(__builtin_rint(rr * a.inv_kc), a.lo_c, a.hi_c);
  tn = (int)t; cn = (int)cc;
}

// Running extremes of a 32-bit v (its |maximum| is folded into the tensor's 64-bit maximum at the end of a tile).
struct VTrack { int vmx, vmn; };
__device__ __forceinline__ void track_v(VTrack& t, int v) { t.vmx = v > t.vmx ? v : t.vmx; t.vmn = v < t.vmn ? v : t.vmn; }
__device__ __forceinline__ uint64_t vtrack_max(const VTrack& t)
{
  const int64_t a = t.vmx, b = -(int64_t)t.vmn;
  return (uint64_t)(a > b ? a : b);
}

// int: theta's grid fixed, 1 <= d, |v| + 2^(d-1) < 2^31 shown by the caller.  RNE(v / 2^d) by add-and-shift.
struct Alg1Int { int d, half_m1, qmin_t, qmax_t, qmin_c, qmax_c; };         // half_m1 = 2^(d-1) - 1

__device__ __forceinline__ void alg1_int(const Alg1Int& a, int v, int& tn, int& cn)
{
  const int q = (v + a.half_m1 + ((v >> a.d) & 1)) >> a.d;
  tn = min(max(q, a.qmin_t), a.qmax_t);
  cn = min(max(v - (int)((unsigned)tn << a.d), a.qmin_c), a.qmax_c);
}

// small: int8 theta, theta's grid fixed, |v| plus the rounding addend below 2^22 (int8 accumulator, d <= 8) or
// 2^23 (int16 accumulator, d <= 22: BIGD).  v is exact in fp32; with M = 1.5 * 2^23 (ulp 1), fma(v, 2^-d, M) is
// M + RNE(v / 2^d) after its single IEEE rounding, clamped as a float between M + qmin and M + qmax.  The low 24
// bits of that float are 2^22 + theta', so one 24-bit multiply-add forms v - theta' * 2^d - 2^(22 + d); the
// accumulator rails are shifted by the same constant, and the low bytes of both results are the bytes to store.
// BIGD: (2^22 + theta') * 2^d no longer fits 32 bits, so theta' is first taken out of the float's bit pattern and
// the residual is formed and clamped unshifted.  tn holds theta' in its LOW BYTE only.
struct Alg1Small { float inv2d_f, lo_tf, hi_tf; int neg2d, lo_cb, hi_cb, lo_c, hi_c; };

__device__ __forceinline__ Alg1Small make_alg1_small(int d, int qmin_t, int qmax_t, int qmin_c, int qmax_c)
{
  Alg1Small a;
  a.inv2d_f = __uint_as_float((uint32_t)(127 - d) << 23);
  a.lo_tf = 12582912.0f + (float)qmin_t; a.hi_tf = 12582912.0f + (float)qmax_t;
  a.neg2d = -(1 << d);
  a.lo_c = qmin_c; a.hi_c = qmax_c;
  a.lo_cb = qmin_c - (1 << (22 + (d <= 8 ? d : 8))); a.hi_cb = qmax_c - (1 << (22 + (d <= 8 ? d : 8)));
  return a;
}

template <bool BIGD>
__device__ __forceinline__ void alg1_small(const Alg1Small& a, int v, int& tn, int& cn)
{
  tn = __float_as_int(__builtin_amdgcn_fmed3f(__builtin_fmaf((float)v, a.inv2d_f, 12582912.0f), a.lo_tf, a.hi_tf));
  if (BIGD) cn = med3_i32(mad_i24(tn - 0x4B400000, a.neg2d, v), a.lo_c, a.hi_c);        // 0x4B400000 = bits(1.5 * 2^23)
  else      cn = med3_i32(mad_i24(tn, a.neg2d, v), a.lo_cb, a.hi_cb);
}

// ---------------------------------------------------------------- stores that skip unchanged data
//
// A lane compares the group it is about to store with the group it loaded.  The wave then decides together: no
// lane saw a change -> no store is issued at all; a few did -> those lanes store, together with the lanes that
// share an aligned LPK_GRANULE-byte run with them (lone 8- or 16-byte writes cost the memory system far more
// than their size); more than half the wave would store -> every lane does, so that HBM sees whole lines.
// Returns true when the store went out dense (every lane).
#ifndef LPK_GRANULE
#define LPK_GRANULE 64        // bytes: the lanes that share such an aligned run of a wave's store go out together
#endif

// Spread each set bit of a lane mask over its aligned group of GL lanes (GL = 1, 2, 4, 8 or 16).
template <int GL> __device__ __forceinline__ uint64_t spread_groups(uint64_t m)
{
  if (GL >= 2)  m |= ((m >> 1) & 0x5555555555555555ull) | ((m & 0x5555555555555555ull) << 1);
  if (GL >= 4)  m |= ((m >> 2) & 0x3333333333333333ull) | ((m & 0x3333333333333333ull) << 2);
  if (GL >= 8)  m |= ((m >> 4) & 0x0f0f0f0f0f0f0f0full) | ((m & 0x0f0f0f0f0f0f0f0full) << 4);
  if (GL >= 16) m |= ((m >> 8) & 0x00ff00ff00ff00ffull) | ((m & 0x00ff00ff00ff00ffull) << 8);
  return m;
}

// LANE_BYTES: bytes one lane stores.  Sparse: only the changed lanes and their neighbours inside the same
// LPK_GRANULE-byte run store, so that memory sees whole granules rather than lone 8- or 16-byte writes.
template <int LANE_BYTES, typename StoreFn>
__device__ __forceinline__ bool lazy_store(bool changed, StoreFn store)
{
  constexpr int GL = LPK_GRANULE / LANE_BYTES > 1 ? LPK_GRANULE / LANE_BYTES : 1;
  uint64_t m = __builtin_amdgcn_ballot_w64(changed);
  if (m == 0) return false;
  m = spread_groups<GL>(m);
  if (__builtin_popcountll(m) * 2 > kWave) { store(); return true; }       // more than half the wave: whole lines
  const int lane = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
  if ((m >> lane) & 1ull) store();
  return false;
}

template <int N> __device__ __forceinline__ bool st_dw_lazy(void* p, const DW<N>& o, const DW<N>& in)
{
  int x = 0;
#pragma unroll
  for (int k = 0; k < N; ++k) x |= o.d[k] ^ in.d[k];
  return lazy_store<4 * N>(x != 0, [&] { st_dw(p, o); });
}

}  // namespace lpk

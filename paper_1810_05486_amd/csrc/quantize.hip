// Uniform linear quantization of fp32 tensors onto a dynamic fixed-point grid,
// round-to-nearest-even, no stochastic rounding (paper, Section 1):
//   q = sat_W(RNE(x * 2^fl)).
//
// 2^fl is an exact fp32 for fl in [-64, 64], so x * 2^fl is exact unless it
// overflows (then it is +-inf and saturates, as the definition does) or falls
// below 2^-126 (then it rounds to 0, as the definition does).  v_rndne_f32
// rounds half to even.  Each lane converts 4 consecutive elements per pass:
// one fully coalesced dwordx4 load, one coalesced 8- or 4-byte store.
//
// Selection and quantization in one pass over the fp32 data (lpk_select_quantize): the exponent of a tensor's
// maximum rarely changes from one training step to the next (Section 6 mentions choosing it from the history of
// maxima for that reason), so the pass quantizes with the fraclen the caller expects -- last step's -- while it
// scans for the maximum, a small kernel derives the true fraclen from the maximum, and only tensors whose guess was
// wrong are quantized again.  The result is the scan's, exactly; the second read of the fp32 data (4 of the 10 bytes
// per element of select-then-quantize) is what disappears.  A tensor that fits one tile is held by one wave, which
// finds its maximum first and quantizes with the true fraclen straight away.
#include "lpk_device.hpp"

namespace lpk {

typedef float    v4f __attribute__((ext_vector_type(4)));
typedef unsigned v2u __attribute__((ext_vector_type(2)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int quant1(float x, float scale, float lo, float hi, bool& nonfinite, uint32_t& ab_max)
{
  const uint32_t ab = __float_as_uint(x) & 0x7fffffffu;
  ab_max = ab > ab_max ? ab : ab_max;              // dead code where the caller does not use the maximum
  if (ab >= 0x7f800000u) nonfinite = true;
  float y = __builtin_rintf(x * scale);
  y = __builtin_fminf(__builtin_fmaxf(y, lo), hi);
  int q = (int)y;
  return ab > 0x7f800000u ? 0 : q;                     // NaN -> 0
}

// E = 4 (int16 out: 8-byte store, int8 out: 4-byte store) or E = 8 (int16: 16-byte store, int8: 8-byte store)
// consecutive elements per lane; KP such groups in flight.
template <int W, int E, int KP>
__device__ __forceinline__ void quant_tile(const float* src, void* dst, bool vec, uint64_t off, uint32_t cnt, float scale, int lane, bool& nf,
                                           uint32_t& ab_max)
{
  const float lo = -(float)(1 << (W - 1)), hi = (float)((1 << (W - 1)) - 1);
  uint32_t done = 0;
  if (vec) {
    const uint32_t ng = cnt / E;
    auto convert_store = [&](const v4f (&x)[E / 4], uint64_t e) {
      int q[E];
#pragma unroll
      for (int k = 0; k < E; ++k) q[k] = quant1(x[k >> 2][k & 3], scale, lo, hi, nf, ab_max);
      uint32_t o[E * W / 32];
#pragma unroll
      for (int w = 0; w < E * W / 32; ++w) {
        if (W == 16) o[w] = (uint32_t)(q[2 * w] & 0xffff) | ((uint32_t)q[2 * w + 1] << 16);
        else o[w] = (uint32_t)(q[4 * w] & 0xff) | ((uint32_t)(q[4 * w + 1] & 0xff) << 8) | ((uint32_t)(q[4 * w + 2] & 0xff) << 16) | ((uint32_t)q[4 * w + 3] << 24);
      }
      char* d = (char*)dst + e * (W / 8);
      if constexpr (E * W / 32 == 1) LPK_STNT(o[0], (LPK_GLOBAL uint32_t*)d);
      else if constexpr (E * W / 32 == 2) { v2u v; v[0] = o[0]; v[1] = o[1]; LPK_STNT(v, (LPK_GLOBAL v2u*)d); }
      else { v4u v; v[0] = o[0]; v[1] = o[1]; v[2] = o[2]; v[3] = o[3]; LPK_STNT(v, (LPK_GLOBAL v4u*)d); }
    };
    uint32_t gi = lane;
    for (; gi + (KP - 1) * kWave < ng; gi += KP * kWave) {
      v4f x[KP][E / 4];
#pragma unroll
      for (int k = 0; k < KP; ++k)
#pragma unroll
        for (int j = 0; j < E / 4; ++j)
          x[k][j] = LPK_LDNT((const LPK_GLOBAL v4f*)(src + off + (uint64_t)(gi + k * kWave) * E + 4 * j));
#pragma unroll
      for (int k = 0; k < KP; ++k) convert_store(x[k], off + (uint64_t)(gi + k * kWave) * E);
    }
    for (; gi < ng; gi += kWave) {
      v4f x[E / 4];
#pragma unroll
      for (int j = 0; j < E / 4; ++j) x[j] = LPK_LDNT((const LPK_GLOBAL v4f*)(src + off + (uint64_t)gi * E + 4 * j));
      convert_store(x, off + (uint64_t)gi * E);
    }
    done = ng * E;
  }
  for (uint32_t j = done + lane; j < cnt; j += kWave) {
    int q = quant1(src[off + j], scale, lo, hi, nf, ab_max);
    if (W == 16) ((int16_t*)dst)[off + j] = (int16_t)q; else ((int8_t*)dst)[off + j] = (int8_t)q;
  }
}

__global__ void __launch_bounds__(kBlock)
quantize_kernel(const TensorDev* __restrict__ tensors, const Tile* __restrict__ tiles, uint32_t n_tiles, int to_theta,
                const int32_t* __restrict__ fl, uint32_t* status)
{
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = wave_uniform(threadIdx.x >> 6);
  const uint32_t w0 = blockIdx.x * kWavesPerBlock + wave;
  const uint32_t nw = gridDim.x * kWavesPerBlock;
  bool nf = false;
  uint32_t bits = 0, unused_max = 0;

  for (uint32_t ti = w0; ti < n_tiles; ti += nw) {
    int t; uint32_t cnt; uint64_t off;
    read_tile(tiles, ti, t, cnt, off);
    const TensorDev T = tensors[t];
    const int f = fl[t];
    if (f < kFlMin || f > kFlMax) { bits |= kStatusDomain; continue; }
    const float scale = __uint_as_float((uint32_t)(127 + f) << 23);           // 2^f, exact
    void* dst = to_theta ? T.theta : T.grad;
    const int W = to_theta ? T.wt : T.wg;
    const bool vec = to_theta ? T.vec_src_theta : T.vec_src_grad;
    if (W == 16) quant_tile<16, LPK_Q_E, LPK_Q_GROUPS>((const float*)T.src, dst, vec, off, cnt, scale, lane, nf, unused_max);
    else         quant_tile<8, LPK_Q_E, LPK_Q_GROUPS>((const float*)T.src, dst, vec, off, cnt, scale, lane, nf, unused_max);
  }
  if (__ballot(nf)) bits |= kStatusNonFinite;
  if (status && bits && lane == 0) atomicOr(status, bits);
}

// ---------------------------------------------------------------- selection and quantization in one pass

__device__ __forceinline__ bool fl_in_domain(int f) { return f >= kFlMin && f <= kFlMax; }

__device__ __forceinline__ void quant_tile_any(int W, const float* src, void* dst, bool vec, uint64_t off, uint32_t cnt, int f, int lane,
                                               bool& nf, uint32_t& ab_max)
{
  const float scale = __uint_as_float((uint32_t)(127 + f) << 23);
  if (W == 16) quant_tile<16, LPK_Q_E, LPK_Q_GROUPS>(src, dst, vec, off, cnt, scale, lane, nf, ab_max);
  else         quant_tile<8, LPK_Q_E, LPK_Q_GROUPS>(src, dst, vec, off, cnt, scale, lane, nf, ab_max);
}

// Pass 1.  A tensor of one tile: maximum, true fraclen (written to fl_out), quantization, all by the wave that holds
// it.  Longer tensors: quantization with the guessed fraclen (none if the guess is outside the domain) while the
// maximum of |bit pattern| is gathered into scratch[t], as the max-abs scan does.
__global__ void __launch_bounds__(kBlock)
quantize_guess_kernel(const TensorDev* __restrict__ tensors, const Tile* __restrict__ tiles, uint32_t n_tiles, int to_theta,
                      const int32_t* fl_guess, int32_t* fl_out, uint32_t* scratch, uint32_t* redo_any, uint32_t* status)
{
  __shared__ int      s_tensor[kWavesPerBlock];
  __shared__ uint32_t s_max[kWavesPerBlock];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = wave_uniform(threadIdx.x >> 6);
  const uint32_t w0 = blockIdx.x * kWavesPerBlock + wave;
  const uint32_t nw = gridDim.x * kWavesPerBlock;
  if (blockIdx.x == 0 && threadIdx.x == 0) *redo_any = 0;      // armed by pass 2, read by pass 3, both later in the stream
  bool nf = false;
  uint32_t bits = 0, lane_max = 0;
  int cur = -1;

  for (uint32_t ti = w0; ti < n_tiles; ti += nw) {
    int t; uint32_t cnt; uint64_t off;
    read_tile(tiles, ti, t, cnt, off);
    if (t != cur) {
      if (cur >= 0) {
        const uint32_t m = wave_max_u32(lane_max);
        if (lane == 0 && m) atomicMax(&scratch[cur], m);
      }
      lane_max = 0;
      cur = t;
    }
    const TensorDev T = tensors[t];
    void* dst = to_theta ? T.theta : T.grad;
    const int W = to_theta ? T.wt : T.wg;
    const bool vec = to_theta ? T.vec_src_theta : T.vec_src_grad;
    if (T.n <= (uint64_t)kTileElems) {
      const uint32_t* s = (const uint32_t*)T.src;
      uint32_t m = 0;
      for (uint32_t j = lane; j < cnt; j += kWave) { const uint32_t ab = s[j] & 0x7fffffffu; m = ab > m ? ab : m; }
      m = wave_max_u32(m);
      const int f = fraclen_of_f32max(m, W, fl_guess[t], lane == 0 ? status : nullptr);
      if (lane == 0) fl_out[t] = f;
      uint32_t unused_max = 0;
      if (fl_in_domain(f)) quant_tile_any(W, (const float*)T.src, dst, vec, off, cnt, f, lane, nf, unused_max);   // the second read hits the cache
      else bits |= kStatusDomain;                      // an all-zero tensor whose default is out of range
    } else {
      const int f = fl_guess[t];
      if (fl_in_domain(f)) {
        quant_tile_any(W, (const float*)T.src, dst, vec, off, cnt, f, lane, nf, lane_max);
      } else {
        const uint32_t* s = (const uint32_t*)T.src + off;
        for (uint32_t j = lane; j < cnt; j += kWave) { const uint32_t ab = s[j] & 0x7fffffffu; lane_max = ab > lane_max ? ab : lane_max; }
      }
    }
  }
  if (__ballot(nf)) bits |= kStatusNonFinite;
  if (status && bits && lane == 0) atomicOr(status, bits);

  flush_block_u32(scratch, cur, lane_max, lane, wave, s_tensor, s_max);
}

// Pass 2, one thread per tensor: the true fraclen of every tensor longer than a tile, and whether its guess was wrong.
__global__ void __launch_bounds__(kBlock)
verify_guess_kernel(const TensorDev* __restrict__ tensors, uint32_t n_tensors, int to_theta, uint32_t* scratch,
                    const int32_t* fl_guess, int32_t* fl_out, uint32_t* redo, uint32_t* redo_any, uint32_t* status)
{
  const uint32_t t = blockIdx.x * kBlock + threadIdx.x;
  if (t >= n_tensors) return;
  const uint64_t n = tensors[t].n;
  redo[t] = 0;
  if (n == 0) { fl_out[t] = fl_guess[t]; return; }    // an empty tensor keeps the caller's fraclen, as in the scan
  if (n <= (uint64_t)kTileElems) return;               // finished by pass 1
  const uint32_t b = scratch[t];
  scratch[t] = 0;                                      // re-arm for the next call
  const int W = to_theta ? tensors[t].wt : tensors[t].wg;
  const int guess = fl_guess[t];
  const int f = fraclen_of_f32max(b, W, guess, status);
  fl_out[t] = f;
  if (!fl_in_domain(f)) { if (status) atomicOr(status, kStatusDomain); return; }   // all zero, default out of range: not quantized
  if (f != guess) { redo[t] = 1; atomicOr(redo_any, 1u); }
}

// Pass 3: nothing, unless some guess was wrong; then the tiles of those tensors once more with the true fraclen.
__global__ void __launch_bounds__(kBlock)
requantize_kernel(const TensorDev* __restrict__ tensors, const Tile* __restrict__ tiles, uint32_t n_tiles, int to_theta,
                  const int32_t* __restrict__ fl, const uint32_t* __restrict__ redo, const uint32_t* __restrict__ redo_any,
                  uint32_t* status)
{
  if (*redo_any == 0) return;
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = wave_uniform(threadIdx.x >> 6);
  const uint32_t w0 = blockIdx.x * kWavesPerBlock + wave;
  const uint32_t nw = gridDim.x * kWavesPerBlock;
  bool nf = false;
  uint32_t unused_max = 0;
  int cur = -1, f = 0;
  bool again = false;
  for (uint32_t ti = w0; ti < n_tiles; ti += nw) {
    int t; uint32_t cnt; uint64_t off;
    read_tile(tiles, ti, t, cnt, off);
    if (t != cur) { cur = t; again = redo[t] != 0; f = fl[t]; }
    if (!again) continue;
    const TensorDev T = tensors[t];
    quant_tile_any(to_theta ? T.wt : T.wg, (const float*)T.src, to_theta ? T.theta : T.grad,
                   to_theta ? T.vec_src_theta : T.vec_src_grad, off, cnt, f, lane, nf, unused_max);
  }
  if (__ballot(nf) && status && lane == 0) atomicOr(status, kStatusNonFinite);
}

hipError_t launch_select_quantize(const TensorDev* tensors, const Tile* tiles, uint32_t n_tiles, uint32_t n_tensors, uint32_t grid,
                                  int to_theta, const int32_t* fl_guess, int32_t* fl_out, uint32_t* scratch, uint32_t* redo,
                                  uint32_t* redo_any, uint32_t* status, hipStream_t stream)
{
  if (n_tiles)
    hipLaunchKernelGGL(quantize_guess_kernel, dim3(grid), dim3(kBlock), 0, stream, tensors, tiles, n_tiles, to_theta, fl_guess, fl_out,
                       scratch, redo_any, status);
  hipLaunchKernelGGL(verify_guess_kernel, dim3((n_tensors + kBlock - 1) / kBlock), dim3(kBlock), 0, stream, tensors, n_tensors, to_theta,
                     scratch, fl_guess, fl_out, redo, redo_any, status);
  if (n_tiles)
    hipLaunchKernelGGL(requantize_kernel, dim3(grid), dim3(kBlock), 0, stream, tensors, tiles, n_tiles, to_theta, fl_out, redo, redo_any,
                       status);
  return hipGetLastError();
}

hipError_t launch_quantize(const TensorDev* tensors, const Tile* tiles, uint32_t n_tiles, uint32_t grid, int to_theta,
                           const int32_t* fl, uint32_t* status, hipStream_t stream)
{
  if (n_tiles)
    hipLaunchKernelGGL(quantize_kernel, dim3(grid), dim3(kBlock), 0, stream, tensors, tiles, n_tiles, to_theta, fl, status);
  return hipGetLastError();
}

}  // namespace lpk

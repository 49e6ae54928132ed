// Uniform linear quantization of fp32 tensors onto a dynamic fixed-point grid,
// round-to-nearest-even, no stochastic rounding (paper, Section 1):
//   q = sat_W(RNE(x * 2^fl)).
//
// 2^fl is an exact fp32 for fl in [-64, 64], so x * 2^fl is exact unless it
// overflows (then it is +-inf and saturates, as the definition does) or falls
// below 2^-126 (then it rounds to 0, as the definition does).  v_rndne_f32
// rounds half to even.  Each lane converts 4 consecutive elements per pass:
// one fully coalesced dwordx4 load, one coalesced 8- or 4-byte store.
#include "lpk_device.hpp"

namespace lpk {

typedef float    v4f __attribute__((ext_vector_type(4)));
typedef unsigned v2u __attribute__((ext_vector_type(2)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int quant1(float x, float scale, float lo, float hi, bool& nonfinite)
{
  const uint32_t ab = __float_as_uint(x) & 0x7fffffffu;
  if (ab >= 0x7f800000u) nonfinite = true;
  float y = __builtin_rintf(x * scale);
  y = __builtin_fminf(__builtin_fmaxf(y, lo), hi);
  int q = (int)y;
  return ab > 0x7f800000u ? 0 : q;                     // NaN -> 0
}

// E = 4 (int16 out: 8-byte store, int8 out: 4-byte store) or E = 8 (int16: 16-byte store, int8: 8-byte store)
// consecutive elements per lane; KP such groups in flight.
template <int W, int E, int KP>
__device__ __forceinline__ void quant_tile(const float* src, void* dst, bool vec, uint64_t off, uint32_t cnt, float scale, int lane, bool& nf)
{
  const float lo = -(float)(1 << (W - 1)), hi = (float)((1 << (W - 1)) - 1);
  uint32_t done = 0;
  if (vec) {
    const uint32_t ng = cnt / E;
    auto convert_store = [&](const v4f (&x)[E / 4], uint64_t e) {
      int q[E];
#pragma unroll
      for (int k = 0; k < E; ++k) q[k] = quant1(x[k >> 2][k & 3], scale, lo, hi, nf);
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
    int q = quant1(src[off + j], scale, lo, hi, nf);
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
  uint32_t bits = 0;

  for (uint32_t ti = w0; ti < n_tiles; ti += nw) {
    const Tile tl = tiles[ti];
    const int t = wave_uniform((int)tl.tensor);
    const uint32_t cnt = (uint32_t)wave_uniform((int)tl.count);
    const uint64_t off = ((uint64_t)(uint32_t)wave_uniform((int)(tl.offset >> 32)) << 32) | (uint32_t)wave_uniform((int)tl.offset);
    const TensorDev T = tensors[t];
    const int f = fl[t];
    if (f < kFlMin || f > kFlMax) { bits |= kStatusDomain; continue; }
    const float scale = __uint_as_float((uint32_t)(127 + f) << 23);           // 2^f, exact
    void* dst = to_theta ? T.theta : T.grad;
    const int W = to_theta ? T.wt : T.wg;
    const bool vec = to_theta ? T.vec_src_theta : T.vec_src_grad;
    if (W == 16) quant_tile<16, LPK_Q_E, LPK_Q_GROUPS>((const float*)T.src, dst, vec, off, cnt, scale, lane, nf);
    else         quant_tile<8, LPK_Q_E, LPK_Q_GROUPS>((const float*)T.src, dst, vec, off, cnt, scale, lane, nf);
  }
  if (__ballot(nf)) bits |= kStatusNonFinite;
  if (status && bits && lane == 0) atomicOr(status, bits);
}

hipError_t launch_quantize(const TensorDev* tensors, const Tile* tiles, uint32_t n_tiles, uint32_t grid, int to_theta,
                           const int32_t* fl, uint32_t* status, hipStream_t stream)
{
  if (n_tiles)
    hipLaunchKernelGGL(quantize_kernel, dim3(grid), dim3(kBlock), 0, stream, tensors, tiles, n_tiles, to_theta, fl, status);
  return hipGetLastError();
}

}  // namespace lpk

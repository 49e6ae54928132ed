// Fractional length per tensor from a max-abs reduction (paper, Section 6: the
// exponent follows the scanned maximum of the tensor; Section 1: dynamic fixed
// point).  Rule: the largest fl at which the maximum still rounds to a code
// <= qmax, i.e. the finest grid on which the tensor's own maximum does not
// saturate.
//
// fp32 source: |x| of a finite float is ordered like its bit pattern with the
// sign cleared, and every NaN/Inf pattern is >= 0x7f800000, so the reduction is
// an unsigned integer max over (bits & 0x7fffffff): per-lane max, DPP wave max,
// LDS across the waves of a block, one atomic per (block, tensor).  Each maximum
// becomes a fraclen in closed form, and its scratch word is re-armed for the
// next call: in the scan's last workgroup when the launch is small, in a second
// small kernel otherwise.
#include "lpk_device.hpp"

namespace lpk {

typedef unsigned v4u __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t absbits(uint32_t b) { return b & 0x7fffffffu; }

// What the scan's last workgroup needs to finish the selection (arrivals == nullptr: a second kernel does it).
struct SelectFold {
  uint32_t*      arrivals;
  uint32_t       n_tensors;
  int            sel;
  const int32_t* fl_default;
  int32_t*       fl_out;
  uint32_t*      status;
};

__global__ void __launch_bounds__(kBlock)
maxabs_f32_kernel(const TensorDev* __restrict__ tensors, const Tile* __restrict__ tiles, uint32_t n_tiles, uint32_t* scratch,
                  SelectFold fold)
{
  __shared__ int      s_tensor[kWavesPerBlock];
  __shared__ uint32_t s_max[kWavesPerBlock];

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = wave_uniform(threadIdx.x >> 6);
  const uint32_t w0 = blockIdx.x * kWavesPerBlock + wave;
  const uint32_t nw = gridDim.x * kWavesPerBlock;

  int cur = -1;
  uint32_t lane_max = 0;
  const float* src = nullptr;
  bool vec = false;

  for (uint32_t ti = w0; ti < n_tiles; ti += nw) {
    int t; uint32_t cnt; uint64_t off;
    read_tile(tiles, ti, t, cnt, off);
    if (t != cur) {
      if (cur >= 0) {
        uint32_t m = wave_max_u32(lane_max);
        if (lane == 0 && m) atomicMax(&scratch[cur], m);
      }
      lane_max = 0;
      cur = t;
      src = (const float*)tensors[t].src;
      vec = (((uintptr_t)src) & 15u) == 0;
    }
    const uint32_t* s = (const uint32_t*)src + off;
    if (vec) {
      // max is order-free: lane l takes the 16-byte pieces l, l+64, ... so every load instruction is fully coalesced
      const uint32_t nv = cnt / 4;
      if (nv == kTileElems / 4) {
        v4u a[kTileElems / 4 / kWave];
#pragma unroll
        for (int j = 0; j < kTileElems / 4 / kWave; ++j) a[j] = LPK_LDNT((const v4u*)s + j * kWave + lane);
#pragma unroll
        for (int j = 0; j < kTileElems / 4 / kWave; ++j) {
          uint32_t m01 = max(absbits(a[j][0]), absbits(a[j][1])), m23 = max(absbits(a[j][2]), absbits(a[j][3]));
          lane_max = max(lane_max, max(m01, m23));
        }
      } else {
        for (uint32_t j = lane; j < nv; j += kWave) {
          v4u a = LPK_LDNT((const v4u*)s + j);
          lane_max = max(lane_max, max(max(absbits(a[0]), absbits(a[1])), max(absbits(a[2]), absbits(a[3]))));
        }
        for (uint32_t j = nv * 4 + lane; j < cnt; j += kWave) lane_max = max(lane_max, absbits(s[j]));
      }
    } else {
      for (uint32_t j = lane; j < cnt; j += kWave) lane_max = max(lane_max, absbits(s[j]));
    }
  }

  flush_block_u32(scratch, cur, lane_max, lane, wave, s_tensor, s_max);

  if (!fold.arrivals) return;
  if (!last_workgroup(fold.arrivals, &s_tensor[0])) return;
  constexpr int K = 4;                                // exchanges in flight per thread
  for (uint32_t base = 0; base < fold.n_tensors; base += K * kBlock) {
    uint32_t b[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const uint32_t t = base + k * kBlock + threadIdx.x;
      b[k] = t < fold.n_tensors ? atomicExch(&scratch[t], 0u) : 0u;     // read, and re-arm for the next call
    }
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const uint32_t t = base + k * kBlock + threadIdx.x;
      if (t >= fold.n_tensors) continue;
      const int W = fold.sel == 1 ? tensors[t].wt : tensors[t].wg;
      fold.fl_out[t] = fraclen_of_f32max(b[k], W, fold.fl_default[t], fold.status);
    }
  }
  if (threadIdx.x == 0) atomicExch(fold.arrivals, 0u);
}

// One thread per tensor: the same conversion as a launch of its own (larger launches; lists without a single element).
__global__ void __launch_bounds__(kBlock)
fraclen_from_f32max_kernel(const TensorDev* __restrict__ tensors, uint32_t n_tensors, int sel,
                           uint32_t* scratch, const int32_t* __restrict__ fl_default, int32_t* fl_out, uint32_t* status)
{
  uint32_t t = blockIdx.x * kBlock + threadIdx.x;
  if (t >= n_tensors) return;
  const uint32_t b = scratch[t];
  scratch[t] = 0;                                   // re-arm for the next call
  const int W = sel == 1 ? tensors[t].wt : tensors[t].wg;
  fl_out[t] = fraclen_of_f32max(b, W, fl_default[t], status);
}


// One thread per tensor: vmax (an integer on grid F = fl_theta_in + d) -> fraclen, clamped to default +- 15.
__global__ void __launch_bounds__(kBlock)
fraclen_from_vmax_kernel(const TensorDev* __restrict__ tensors, uint32_t n_tensors, int sel,
                         const uint64_t* __restrict__ vmax, const int32_t* __restrict__ fl_theta_in,
                         const int32_t* __restrict__ fl_default, int32_t* fl_out, uint32_t* status)
{
  uint32_t t = blockIdx.x * kBlock + threadIdx.x;
  if (t >= n_tensors) return;
  // sel: 0 gradient width, 1 theta width (vmax on grid fl + d), 2 velocity / first-moment width and 3 second-moment
  // width (maxima on the state's own grid)
  const int W = sel == 1 ? tensors[t].wt : (sel == 2 ? tensors[t].wm : (sel == 3 ? tensors[t].wu : tensors[t].wg));
  const int d = sel >= 2 ? 0 : (tensors[t].comp ? tensors[t].d : 0);
  const int F = fl_theta_in[t] + d;
  const int cur = fl_default[t];
  if (F < kFlMin || F > kFlMax + kDMax || cur < kFlMin || cur > kFlMax) {
    fl_out[t] = cur;
    if (status) atomicOr(status, kStatusDomain);
    return;
  }
  const uint64_t v = vmax[t];
  if (v == 0) { fl_out[t] = cur; return; }
  const int e = 63 - __clzll((long long)v);
  int fl = W - 2 - e + F;
  // too fine iff v * 2^(W-2-e) >= 2^(W-1) - 1/2  <=>  v * 2^(W-1-e) >= 2^W - 1
  const uint64_t rail = (1ull << W) - 1ull;
  const int sh = W - 1 - e;
  const bool over = sh >= 0 ? (v << sh) >= rail : v >= (rail << (-sh));     // e <= 63, W <= 16: no overflow either way
  if (over) fl -= 1;
  if (fl > cur + kDeltaMax) fl = cur + kDeltaMax;
  if (fl < cur - kDeltaMax) fl = cur - kDeltaMax;
  fl_out[t] = clamp_fl(fl);
}

// `arrivals`: the list's workgroup counter for this launch (zero between launches), or nullptr to convert in a
// second launch whatever the launch's size.
hipError_t launch_select_f32(const TensorDev* tensors, const Tile* tiles, uint32_t n_tiles, uint32_t n_tensors, uint32_t grid,
                             int sel, uint32_t* scratch, uint32_t* arrivals, const int32_t* fl_default, int32_t* fl_out,
                             uint32_t* status, hipStream_t stream)
{
  const bool fold = arrivals && n_tiles && n_tensors <= kFoldMaxTensors && grid <= kFoldMaxBlocks;
  if (n_tiles) {
    const SelectFold f{fold ? arrivals : nullptr, n_tensors, sel, fl_default, fl_out, status};
    hipLaunchKernelGGL(maxabs_f32_kernel, dim3(grid), dim3(kBlock), 0, stream, tensors, tiles, n_tiles, scratch, f);
  }
  if (!fold)
    hipLaunchKernelGGL(fraclen_from_f32max_kernel, dim3((n_tensors + kBlock - 1) / kBlock), dim3(kBlock), 0, stream,
                     tensors, n_tensors, sel, scratch, fl_default, fl_out, status);
  return hipGetLastError();
}

hipError_t launch_select_vmax(const TensorDev* tensors, uint32_t n_tensors, int sel, const uint64_t* vmax,
                              const int32_t* fl_theta_in, const int32_t* fl_default, int32_t* fl_out, uint32_t* status,
                              hipStream_t stream)
{
  hipLaunchKernelGGL(fraclen_from_vmax_kernel, dim3((n_tensors + kBlock - 1) / kBlock), dim3(kBlock), 0, stream,
                     tensors, n_tensors, sel, vmax, fl_theta_in, fl_default, fl_out, status);
  return hipGetLastError();
}

}  // namespace lpk

// Shared between the host layer and the gfx950 kernels of liblpk: device-side
// tables, launch geometry and wavefront reductions.  Nothing here is used by
// the CPU oracle.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define LPK_GLOBAL __attribute__((address_space(1)))

// Tuning constants of the streaming kernels (overridable at compile time for experiments).
#ifndef LPK_PASSES
#define LPK_PASSES 4          // 1024-element passes per wave tile, all loads of a tile in flight together
#endif
#ifndef LPK_KP_WIDE
#define LPK_KP_WIDE 2         // groups in flight per lane when one group needs more than 16 VGPRs
#endif
#ifndef LPK_F32_E
#define LPK_F32_E 8           // consecutive elements per lane in the fp32-gradient update
#endif
#ifndef LPK_F32_GROUPS
#define LPK_F32_GROUPS 4      // such groups in flight per lane
#endif
#ifndef LPK_I16_E
#define LPK_I16_E 16          // consecutive elements per lane with int16 gradients (16 = the pipelined dwordx4 path)
#endif
#ifndef LPK_I16_GROUPS
#define LPK_I16_GROUPS 4
#endif
// The same three counts for the tile forms that test their stores: a read-mostly stream with scattered writes runs
// 3-7 % faster with two groups in flight than with four (measured at two workgroups per CU).
#ifndef LPK_I16_GROUPS_LAZY
#define LPK_I16_GROUPS_LAZY 2
#endif
#ifndef LPK_I8_E_BOTH
#define LPK_I8_E_BOTH 8       // int16 gradients, 8-bit arrays, form that tests theta's and comp's stores: elements per lane ...
#endif
#ifndef LPK_I8_GROUPS_BOTH
#define LPK_I8_GROUPS_BOTH 4  // ... and groups in flight
#endif
#ifndef LPK_F32_GROUPS_LAZY
#define LPK_F32_GROUPS_LAZY 2
#endif
#ifndef LPK_F32_E_BOTH
#define LPK_F32_E_BOTH 4      // fp32 gradients, form that tests theta's and comp's stores: elements per lane ...
#endif
#ifndef LPK_F32_GROUPS_BOTH
#define LPK_F32_GROUPS_BOTH 8 // ... and groups in flight
#endif
#ifndef LPK_W16_GROUPS_LAZY
#define LPK_W16_GROUPS_LAZY 2
#endif
#ifndef LPK_W16_GROUPS
#define LPK_W16_GROUPS 4      // groups of 8 elements in flight per lane when theta or comp is 16 bits wide
#endif
#ifndef LPK_WAVES_PER_BLOCK
#define LPK_WAVES_PER_BLOCK 4 // wavefronts per workgroup of the persistent kernels
#endif
#ifndef LPK_Q_E
#define LPK_Q_E 4             // consecutive elements per lane in the quantization kernel
#endif
#ifndef LPK_Q_GROUPS
#define LPK_Q_GROUPS 8        // such groups in flight per lane (with one workgroup per CU; measured best of 2-16 x 1-3)
#endif
#ifndef LPK_FOLD_MAX_TENSORS
#define LPK_FOLD_MAX_TENSORS 4096   // lists up to this length (0: none) ...
#endif
#ifndef LPK_FOLD_MAX_BLOCKS
#define LPK_FOLD_MAX_BLOCKS 128     // ... in launches of up to this many workgroups end their maxima in the last workgroup
#endif
#ifndef LPK_NT_LOAD
#define LPK_NT_LOAD 1         // non-temporal hint on streaming loads
#endif
#ifndef LPK_NT_STORE
#define LPK_NT_STORE 1        // non-temporal hint on streaming stores
#endif
#if LPK_NT_LOAD
#define LPK_LDNT(p) __builtin_nontemporal_load(p)
#else
#define LPK_LDNT(p) (*(p))
#endif
#if LPK_NT_STORE
#define LPK_STNT(v, p) __builtin_nontemporal_store(v, p)
#else
#define LPK_STNT(v, p) (*(p) = (v))
#endif

namespace lpk {

constexpr int kWave           = 64;     // CDNA wavefront
constexpr int kWavesPerBlock  = LPK_WAVES_PER_BLOCK;
constexpr int kBlock          = kWave * kWavesPerBlock;
constexpr int kGroup          = 16;     // elements one lane handles per pass (one dwordx4 of int8)
constexpr int kPassElems      = kWave * kGroup;          // 1024 elements per wave pass
constexpr int kPasses         = LPK_PASSES;
constexpr int kTileElems      = kPassElems * kPasses;    // 4096 elements per wave tile

constexpr int kFlMin = -64, kFlMax = 64, kDMax = 24, kDeltaMax = 15;
constexpr uint32_t kStatusNonFinite = 1u, kStatusDomain = 2u;

// One tensor, as the kernels see it (72 bytes, read with scalar loads).
struct TensorDev {
  void*       theta;
  void*       comp;      // nullptr: no accumulator
  void*       grad;
  const void* src;       // fp32 source
  uint64_t    n;
  uint8_t     wt, wc, wg, d;        // widths in bits (wc = 0 without comp), comp shift
  uint8_t     vec_step, vec_src_grad, vec_src_theta, wm;     // 16-byte alignment facts; velocity width (0 = none)
  void*       mom;       // velocity of the momentum update / first moment of ADAM, nullptr = none
  uint8_t     vec_mom, wu, vec_adam, pad0[5];                // wu: width of the second moment (0 = none)
  void*       sec;       // second moment of ADAM, nullptr = none
};
static_assert(sizeof(TensorDev) == 72, "descriptor layout");

// One wave-sized piece of one tensor.
struct Tile {
  uint32_t tensor;
  uint32_t count;        // 1..kTileElems elements
  uint64_t offset;       // first element, a multiple of kTileElems
};
static_assert(sizeof(Tile) == 16, "tile layout");

// Hyper-parameters of the ADAM update as the kernel receives them (by value).
struct AdamHyperDev { uint32_t lr, lr_exp, b1, b2, eps, eps_exp; };

// ---- wavefront max over unsigned 32-bit values, via DPP -------------------
// Row shifts build the maximum of each 16-lane row in its last lane, two row
// broadcasts carry it across rows; lane 63 ends with the wave maximum.
// Out-of-range and masked lanes contribute 0, the identity of unsigned max.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
  uint32_t t;
  t = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, true);  v = v > t ? v : t;   // row_shr:1
  t = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, true);  v = v > t ? v : t;   // row_shr:2
  t = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, true);  v = v > t ? v : t;   // row_shr:4
  t = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, true);  v = v > t ? v : t;   // row_shr:8
  t = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, true);  v = v > t ? v : t;   // row_bcast:15 -> rows 1,3
  t = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, true);  v = v > t ? v : t;   // row_bcast:31 -> rows 2,3
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// 64-bit unsigned wave max: high halves first, then the low halves of the
// lanes that hold the winning high half.
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v)
{
  uint32_t hi = (uint32_t)(v >> 32), lo = (uint32_t)v;
  uint32_t mh = wave_max_u32(hi);
  uint32_t ml = wave_max_u32(hi == mh ? lo : 0u);
  return ((uint64_t)mh << 32) | ml;
}

__device__ __forceinline__ int wave_uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }

// Decode one tile-table entry into wave-uniform scalars.
__device__ __forceinline__ void read_tile(const Tile* __restrict__ tiles, uint32_t ti, int& tensor, uint32_t& cnt, uint64_t& off)
{
  const Tile tl = tiles[ti];
  tensor = wave_uniform((int)tl.tensor);
  cnt = (uint32_t)wave_uniform((int)tl.count);
  off = ((uint64_t)(uint32_t)wave_uniform((int)(tl.offset >> 32)) << 32) | (uint32_t)wave_uniform((int)tl.offset);
}

// Block-level end of a persistent scan: the waves of a block usually end on the same tensor, so their (tensor, max)
// pairs are combined in LDS and each tensor gets one atomic.  s_tensor, s_max: one LDS word per wave each.
__device__ __forceinline__ void flush_block_u32(uint32_t* scratch, int cur, uint32_t lane_max, int lane, int wave,
                                                int* s_tensor, uint32_t* s_max)
{
  const uint32_t m = wave_max_u32(lane_max);
  if (lane == 0) { s_tensor[wave] = cur; s_max[wave] = m; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int a = 0; a < kWavesPerBlock; ++a) {
      const int ta = s_tensor[a];
      if (ta < 0) continue;
      uint32_t ma = s_max[a];
      for (int b = a + 1; b < kWavesPerBlock; ++b)
        if (s_tensor[b] == ta) { ma = ma > s_max[b] ? ma : s_max[b]; s_tensor[b] = -1; }
      if (ma) atomicMax(&scratch[ta], ma);
    }
  }
}

// ---- fraclen of an fp32 maximum ------------------------------------------------
__device__ __forceinline__ int clamp_fl(int fl) { return fl > kFlMax ? kFlMax : (fl < kFlMin ? kFlMin : fl); }

// Max bit pattern of a tensor -> fraclen.  With e = floor(log2 M) the candidate is W - 2 - e (M lands in
// [2^(W-2), 2^(W-1))); it is one too fine exactly when M * 2^fl reaches 2^(W-1) - 1/2, i.e. when the 24-bit
// significand m satisfies m >= 2^24 - 2^(24-W).
__device__ __forceinline__ int fraclen_of_f32max(uint32_t b, int W, int fl_default, uint32_t* status)
{
  if (b >= 0x7f800000u) { if (status) atomicOr(status, kStatusNonFinite); return kFlMin; }
  if (b == 0) return fl_default;
  const int E = (int)(b >> 23);
  if (E == 0) return kFlMax;                          // subnormal maximum: far finer than the domain allows
  const uint32_t m = (b & 0x7fffffu) | 0x800000u;
  int fl = W - 2 - (E - 127);
  if (m >= (1u << 24) - (1u << (24 - W))) fl -= 1;
  return clamp_fl(fl);
}

// ---- ending a launch in its last workgroup ---------------------------------
// Per-tensor maxima are gathered with atomics from every workgroup of a launch.  In small launches (up to
// kFoldMaxBlocks workgroups, lists of up to kFoldMaxTensors tensors) the workgroup that finishes last turns them
// into the call's outputs and re-arms the accumulators, which saves the launches that would otherwise clear before
// and convert after: 5-6 us of the 28-34 us a whole step takes on parameter sets of up to two million elements.
// Nobody waits for anybody: a workgroup counts itself in when its own atomics are performed, and the one that
// counts last does the work.  Counting in costs every workgroup one atomic with a returned value on one shared
// word, which the device serialises (about 10 ns each): at 256 workgroups that has eaten the gain, at 2048 it costs
// 10 us per step, hence the limit.
constexpr uint32_t kFoldMaxTensors = LPK_FOLD_MAX_TENSORS;
constexpr uint32_t kFoldMaxBlocks  = LPK_FOLD_MAX_BLOCKS;

// True in every thread of exactly one workgroup of the launch: the last to get here.  `arrivals` must be 0 when
// the launch starts (the caller of this function puts it back); `s_flag` is one LDS word the block can spare.
//
// Only device-scope read-modify-write atomics carry data between the workgroups here (the maxima, the counter;
// the last workgroup reads with atomic exchanges too), so every access to those words is performed at the one place
// where the device performs its atomics; what has to be added is their order.  vmcnt(0) means that every atomic this
// wave issued has been performed, the barrier extends that to the block, and only then does the block count itself
// in, so the workgroup that reads gridDim.x - 1 reads after every maximum is in.  A device-scope fence is not used:
// on this chip it writes back and invalidates the whole L2 of the XCD, and a few thousand workgroups doing that cost
// four times the step (measured).
__device__ __forceinline__ bool last_workgroup(uint32_t* arrivals, int* s_flag)
{
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0) *s_flag = atomicAdd(arrivals, 1u) == gridDim.x - 1;
  __syncthreads();
  return *s_flag != 0;
}

// Accumulators of up to three per-tensor maxima (in the list's own memory, zero between launches) and where the
// call wants them.  arrivals == nullptr: the kernel's pointers are the outputs themselves, cleared by a launch before.
struct MaxFold {
  uint32_t* arrivals;
  uint32_t  n_tensors;
  uint64_t* out[3];
};

// Host side: where a launch gathers its maxima.  With the list's accumulators (`fold_acc`: three arrays of
// n_tensors words; `arrivals`: its workgroup counter) in a launch small enough, the kernel gathers there and its last
// workgroup fills the outputs; otherwise the kernel gathers in the outputs, which a launch before must clear.
struct MaxPlan { MaxFold fold; uint64_t* acc[3]; };
inline MaxPlan plan_maxima(uint64_t* fold_acc, uint32_t* arrivals, uint32_t n_tensors, uint32_t n_tiles, uint32_t grid,
                           uint64_t* out0, uint64_t* out1, uint64_t* out2)
{
  uint64_t* const out[3] = {out0, out1, out2};
  const bool fold = fold_acc && arrivals && n_tiles && n_tensors <= kFoldMaxTensors && grid <= kFoldMaxBlocks &&
                    (out0 || out1 || out2);
  MaxPlan p{};
  p.fold.arrivals = fold ? arrivals : nullptr;
  p.fold.n_tensors = n_tensors;
  for (int i = 0; i < 3; ++i) {
    p.fold.out[i] = out[i];
    p.acc[i] = !fold ? out[i] : (out[i] ? fold_acc + (size_t)i * n_tensors : nullptr);
  }
  return p;
}

template <int N>
__device__ __forceinline__ void fold_maxima(const MaxFold& f, uint64_t* const (&acc)[N], int* s_flag)
{
  if (!last_workgroup(f.arrivals, s_flag)) return;
  constexpr int K = 4;                   // exchanges in flight per thread and array
  for (uint32_t base = 0; base < f.n_tensors; base += K * kBlock) {
    uint64_t v[N][K];
#pragma unroll
    for (int a = 0; a < N; ++a)
#pragma unroll
      for (int k = 0; k < K; ++k) {
        const uint32_t t = base + k * kBlock + threadIdx.x;
        v[a][k] = 0;
        if (acc[a] && t < f.n_tensors)   // read and re-arm in one atomic
          v[a][k] = atomicExch((unsigned long long*)&acc[a][t], 0ull);
      }
#pragma unroll
    for (int a = 0; a < N; ++a)
#pragma unroll
      for (int k = 0; k < K; ++k) {
        const uint32_t t = base + k * kBlock + threadIdx.x;
        if (acc[a] && t < f.n_tensors) f.out[a][t] = v[a][k];
      }
  }
  if (threadIdx.x == 0) atomicExch(f.arrivals, 0u);
}

}  // namespace lpk

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

}  // namespace lpk

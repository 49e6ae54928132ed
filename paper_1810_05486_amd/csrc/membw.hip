// libmembw: memory-system yardsticks for the benchmark -- NOT part of liblpk or of its C ABI.
//
// Each "mix" is the HBM access pattern of one of the library's streaming kernels with the arithmetic taken out:
// the same arrays, the same bytes per lane and access, the same in-place read-modify-write or out-of-place
// structure, the same persistent grid of wavefronts walking tiles, the same non-temporal 16-byte global accesses.
// What a mix reaches is what the memory system gives that traffic; a kernel is read against it, next to the
// 8 TB/s peak.  The plain copy also calibrates the profiler's FETCH_SIZE / WRITE_SIZE counters (known bytes).
//
// A unit is what one lane handles per pass: 16 parameters.  An array holds `words` 16-byte words per unit
// (1 = an int8 array, 2 = int16, 4 = fp32) and is read, written, or read and written back in place.  Two lane
// layouts: "coalesced" (every access instruction of a wave covers one contiguous 1 KiB run: lane l takes words
// l, l + 64, ... of the wave's piece of the array -- the friendliest form for the memory system, the one the table
// of ceilings uses) and "lane-consecutive" (a lane's words are adjacent in memory, so a wave's access has a stride of
// words * 16 bytes between lanes -- what a kernel does when one lane owns 16 consecutive parameters of every
// array).  A third layout halves the unit to 8 parameters per lane ("half units": an int8 array is then read and
// written 8 bytes per lane, a 16-bit one 16 bytes per lane, coalesced) -- the shape of the kernels whose state
// includes a 16-bit array.  `groups` passes of a wave are in flight together: all their loads are issued before the
// first store, as in the update kernels.
//
// `work` > 0 puts that many dependent fp32 multiply-adds per parameter between a pass's loads and its stores (four
// independent chains per lane; the stored words depend on their results): the same traffic with a kernel's amount
// of arithmetic in between, to tell what the arithmetic's mere presence costs a stream that is not bound by it.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#define MEMBW_GLOBAL __attribute__((address_space(1)))

namespace {

typedef unsigned v4u __attribute__((ext_vector_type(4)));

constexpr int kWave = 64, kWavesPerBlock = 4, kBlock = kWave * kWavesPerBlock, kMaxArrays = 8;
enum { kRead = 1, kWrite = 2, kReadWrite = 3 };

struct Ptrs { v4u* a[kMaxArrays]; };

// WM...: per array, words * 4 + mode.
template <int... WM> struct Mix {
  static constexpr int n = sizeof...(WM);
  static constexpr int code[sizeof...(WM)] = {WM...};
  static constexpr int total_words() { int t = 0; for (int i = 0; i < n; ++i) t += code[i] >> 2; return t; }
};

typedef unsigned v2u __attribute__((ext_vector_type(2)));

// One lane's share of one array in one pass, as up to four 16-byte registers.
//   LAYOUT 0 (coalesced): words k * 64 + lane of the pass's piece of the array, k < words.
//   LAYOUT 1 (lane-consecutive): words lane * words + k.
//   LAYOUT 2 (half units, 8 parameters per lane): an array of `words` words per 16 parameters holds words * 8 bytes
//     per lane: one 8-byte access when words == 1, else words / 2 coalesced 16-byte accesses.
template <int LAYOUT>
__device__ __forceinline__ void load_share(v4u (&r)[4], const v4u* base, uint64_t ub, int lane, int words)
{
  if (LAYOUT == 2) {
    if (words == 1) {
      const v2u x = __builtin_nontemporal_load((const MEMBW_GLOBAL v2u*)((const v2u*)base + ub + lane));
      r[0] = v4u{x[0], x[1], 0u, 0u};
    } else {
#pragma unroll
      for (int k = 0; k < words / 2; ++k)
        r[k] = __builtin_nontemporal_load((const MEMBW_GLOBAL v4u*)(base + ub * (words / 2) + (uint64_t)k * kWave + lane));
    }
    return;
  }
#pragma unroll
  for (int k = 0; k < words; ++k)
    r[k] = __builtin_nontemporal_load((const MEMBW_GLOBAL v4u*)(base + (LAYOUT == 0 ? ub * words + (uint64_t)k * kWave + lane : (ub + lane) * words + k)));
}

template <int LAYOUT>
__device__ __forceinline__ void store_share(const v4u (&r)[4], v4u* base, uint64_t ub, int lane, int words)
{
  if (LAYOUT == 2) {
    if (words == 1) {
      __builtin_nontemporal_store(v2u{r[0][0], r[0][1]}, (MEMBW_GLOBAL v2u*)((v2u*)base + ub + lane));
    } else {
#pragma unroll
      for (int k = 0; k < words / 2; ++k)
        __builtin_nontemporal_store(r[k], (MEMBW_GLOBAL v4u*)(base + ub * (words / 2) + (uint64_t)k * kWave + lane));
    }
    return;
  }
#pragma unroll
  for (int k = 0; k < words; ++k)
    __builtin_nontemporal_store(r[k], (MEMBW_GLOBAL v4u*)(base + (LAYOUT == 0 ? ub * words + (uint64_t)k * kWave + lane : (ub + lane) * words + k)));
}

template <typename M, int KP, int LAYOUT>
__global__ void __launch_bounds__(kBlock) membw_kernel(Ptrs p, uint64_t n_tiles, unsigned* sink, int work)
{
  const int lane = threadIdx.x & (kWave - 1);
  const uint64_t w0 = (uint64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6), nw = (uint64_t)gridDim.x * kWavesPerBlock;
  v4u acc = {0u, 0u, 0u, 0u};
  for (uint64_t t = w0; t < n_tiles; t += nw) {
    v4u r[KP][M::n][4];
#pragma unroll
    for (int ps = 0; ps < KP; ++ps) {
      const uint64_t ub = (t * KP + ps) * kWave;
#pragma unroll
      for (int i = 0; i < M::n; ++i) {
        const int words = M::code[i] >> 2, mode = M::code[i] & 3;
#pragma unroll
        for (int k = 0; k < 4; ++k) r[ps][i][k] = v4u{0u, 0u, 0u, 0u};
        if (mode & kRead) load_share<LAYOUT>(r[ps][i], p.a[i], ub, lane, words);
      }
    }
#pragma unroll
    for (int ps = 0; ps < KP; ++ps) {
      const uint64_t ub = (t * KP + ps) * kWave;
      v4u ro = {(unsigned)lane, 0u, 0u, 0u};                  // what the written words depend on: every read-only word
#pragma unroll
      for (int i = 0; i < M::n; ++i) {
        if ((M::code[i] & 3) == kRead) {
#pragma unroll
          for (int k = 0; k < 4; ++k) ro ^= r[ps][i][k];
        }
      }
      if (work > 0) {
        float f0 = (float)(ro[0] & 0xffu), f1 = (float)(ro[1] & 0xffu), f2 = (float)(ro[2] & 0xffu), f3 = (float)(ro[3] & 0xffu);
        for (int w = 0; w < 4 * work; ++w) {                  // 16 parameters per lane and pass, four multiply-adds per turn
          f0 = __builtin_fmaf(f0, 0.5f, 1.0f); f1 = __builtin_fmaf(f1, 0.25f, 3.0f);
          f2 = __builtin_fmaf(f2, 0.75f, 5.0f); f3 = __builtin_fmaf(f3, 0.125f, 7.0f);
        }
        ro ^= v4u{__float_as_uint(f0), __float_as_uint(f1), __float_as_uint(f2), __float_as_uint(f3)};
      }
      acc ^= ro;
#pragma unroll
      for (int i = 0; i < M::n; ++i) {
        const int words = M::code[i] >> 2, mode = M::code[i] & 3;
        if (mode & kWrite) {
          v4u o[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) o[k] = mode == kReadWrite ? (r[ps][i][k] ^ ro) : ro;
          store_share<LAYOUT>(o, p.a[i], ub, lane, words);
        }
      }
    }
  }
  // keeps the loads of a read-only mix alive; the condition is never true for the data the benchmark uses
  if (sink && (acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u && n_tiles == ~0ull) *sink = acc[0];
}

struct MixInfo { const char* name; int n; int words[kMaxArrays]; int modes[kMaxArrays]; };

#define W(words, mode) ((words) * 4 + (mode))
typedef Mix<W(1, kRead)>                                                        MixRead;
typedef Mix<W(1, kWrite)>                                                       MixWrite;
typedef Mix<W(1, kRead), W(1, kWrite)>                                          MixCopy;
typedef Mix<W(1, kReadWrite), W(1, kReadWrite), W(2, kRead)>                    MixUpdate8;     // int8 theta, comp; int16 grad
typedef Mix<W(1, kReadWrite), W(1, kReadWrite), W(1, kReadWrite), W(2, kRead)>  MixMomentum8;   // + int8 velocity
typedef Mix<W(1, kReadWrite), W(1, kReadWrite), W(2, kReadWrite), W(2, kRead)>  MixMomentum16;  // + int16 velocity
typedef Mix<W(1, kReadWrite), W(1, kReadWrite), W(2, kReadWrite), W(2, kReadWrite), W(2, kRead)> MixAdam;   // + two int16 moments
typedef Mix<W(4, kRead), W(2, kWrite)>                                          MixQuantize;    // fp32 in, int16 out
typedef Mix<W(2, kReadWrite), W(2, kReadWrite), W(2, kRead)>                    MixUpdate16;    // int16 theta, comp, grad
typedef Mix<W(1, kReadWrite), W(1, kReadWrite), W(4, kRead)>                    MixUpdateF32;   // int8 theta, comp; fp32 grad
typedef Mix<W(1, kReadWrite), W(2, kReadWrite), W(2, kRead)>                    MixUpdate8C16;  // int8 theta, int16 comp
#undef W

template <typename M> MixInfo info_of(const char* name)
{
  MixInfo m{name, M::n, {}, {}};
  for (int i = 0; i < M::n; ++i) { m.words[i] = M::code[i] >> 2; m.modes[i] = M::code[i] & 3; }
  return m;
}

const MixInfo kMixes[] = {
  info_of<MixRead>("read"), info_of<MixWrite>("write"), info_of<MixCopy>("copy"),
  info_of<MixUpdate8>("update_i8 (4R:2W in place)"), info_of<MixMomentum8>("momentum_i8v (5R:3W in place)"),
  info_of<MixMomentum16>("momentum_i16v (6R:4W in place)"), info_of<MixAdam>("adam_i16 (8R:6W in place)"),
  info_of<MixQuantize>("quantize (4R:2W out of place)"), info_of<MixUpdate16>("update_i16 (6R:4W in place)"),
  info_of<MixUpdateF32>("update_f32grad (6R:2W in place)"), info_of<MixUpdate8C16>("update_i8_c16 (5R:3W in place)"),
};
constexpr int kNumMixes = sizeof(kMixes) / sizeof(kMixes[0]);

// n_units: units of 16 parameters; a pass of the half-unit layout covers 64 * 8 parameters, the others 64 * 16.
template <typename M, int C>
hipError_t launch(int groups, uint32_t grid, const Ptrs& p, uint64_t n_units, unsigned* sink, int work, hipStream_t s)
{
  const uint64_t n_tiles = (C == 2 ? 2 * n_units : n_units) / ((uint64_t)groups * kWave);
  if (n_tiles == 0) return hipSuccess;
  if (grid > (n_tiles + kWavesPerBlock - 1) / kWavesPerBlock) grid = (uint32_t)((n_tiles + kWavesPerBlock - 1) / kWavesPerBlock);
  switch (groups) {
    case 1: hipLaunchKernelGGL((membw_kernel<M, 1, C>), dim3(grid), dim3(kBlock), 0, s, p, n_tiles, sink, work); break;
    case 2: hipLaunchKernelGGL((membw_kernel<M, 2, C>), dim3(grid), dim3(kBlock), 0, s, p, n_tiles, sink, work); break;
    case 4: hipLaunchKernelGGL((membw_kernel<M, 4, C>), dim3(grid), dim3(kBlock), 0, s, p, n_tiles, sink, work); break;
    case 8: hipLaunchKernelGGL((membw_kernel<M, 8, C>), dim3(grid), dim3(kBlock), 0, s, p, n_tiles, sink, work); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace

extern "C" {

int membw_mix_count(void) { return kNumMixes; }

// Name, array count, words per unit and mode (1 read, 2 write, 3 read + write in place) of every array of a mix.
// Returns the array count, or -1 for an unknown mix.
int membw_mix_describe(int mix, char* name, int name_cap, int* words, int* modes)
{
  if (mix < 0 || mix >= kNumMixes) return -1;
  const MixInfo& m = kMixes[mix];
  if (name && name_cap > 0) { strncpy(name, m.name, (size_t)name_cap - 1); name[name_cap - 1] = 0; }
  for (int i = 0; i < m.n; ++i) { if (words) words[i] = m.words[i]; if (modes) modes[i] = m.modes[i]; }
  return m.n;
}

// Run one mix over n_units units (rounded down to whole tiles of groups * 64 units; every access stays inside the
// first n_units * words * 16 bytes of each array).  arrays: host array of device pointers, one per array of the
// mix, each 16-byte aligned and at least n_units * words * 16 bytes long, not overlapping.  groups in {1, 2, 4, 8};
// blocks_per_cu >= 1; layout 0 = coalesced, 1 = lane-consecutive, 2 = half units (8 parameters per lane); work: fp32
// multiply-adds per parameter between loads and stores, 0..4096 (in the half-unit layout a pass holds half the
// parameters, so the count per parameter is twice `work`).  Only enqueues.
// Returns 0, or -1 for a bad argument, -3 for a HIP failure.
int membw_run_work(int mix, int groups, int blocks_per_cu, int layout, void* const* arrays, uint64_t n_units, int work,
                   void* stream)
{
  if (mix < 0 || mix >= kNumMixes || !arrays || blocks_per_cu < 1 || blocks_per_cu > 64 || work < 0 || work > 4096) return -1;
  if ((groups != 1 && groups != 2 && groups != 4 && groups != 8) || layout < 0 || layout > 2) return -1;
  Ptrs p{};
  for (int i = 0; i < kMixes[mix].n; ++i) {
    if (!arrays[i] || ((uintptr_t)arrays[i] & 15u)) return -1;
    p.a[i] = (v4u*)arrays[i];
  }
  int dev = 0, n_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
    return -3;
  const uint32_t grid = (uint32_t)n_cu * (uint32_t)blocks_per_cu;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = hipErrorInvalidValue;
#define MEMBW_CASE(id, M) case id: e = layout == 0 ? launch<M, 0>(groups, grid, p, n_units, nullptr, work, s) : (layout == 1 ? launch<M, 1>(groups, grid, p, n_units, nullptr, work, s) : launch<M, 2>(groups, grid, p, n_units, nullptr, work, s)); break
  switch (mix) {
    MEMBW_CASE(0, MixRead);
    MEMBW_CASE(1, MixWrite);
    MEMBW_CASE(2, MixCopy);
    MEMBW_CASE(3, MixUpdate8);
    MEMBW_CASE(4, MixMomentum8);
    MEMBW_CASE(5, MixMomentum16);
    MEMBW_CASE(6, MixAdam);
    MEMBW_CASE(7, MixQuantize);
    MEMBW_CASE(8, MixUpdate16);
    MEMBW_CASE(9, MixUpdateF32);
    MEMBW_CASE(10, MixUpdate8C16);
    default: break;
  }
#undef MEMBW_CASE
  return e == hipSuccess ? 0 : -3;
}

// The plain yardstick: no arithmetic between loads and stores.
int membw_run(int mix, int groups, int blocks_per_cu, int layout, void* const* arrays, uint64_t n_units, void* stream)
{
  return membw_run_work(mix, groups, blocks_per_cu, layout, arrays, n_units, 0, stream);
}

}  // extern "C"

// lpk_kahan_sgd_step_noalloc: the lazy update for callers that cannot allocate device memory (code under HIP
// graph capture, tight serving loops, harnesses that forbid hipMalloc).  It takes the caller's descriptors
// directly instead of a list made by lpk_tensor_list_create, and keeps what that call would have allocated -- the
// kernels' descriptor table and the tile table -- in a file-scope device array of fixed size.
//
// The tables travel to the device as kernel arguments: a staging kernel receives up to kChunk descriptors by
// value, writes them into the table and cuts each of those tensors into tiles on the device.  Nothing is copied
// from host memory asynchronously, nothing is allocated, nothing synchronizes; the update kernels then run on the
// same stream exactly as lpk_kahan_sgd_step runs them.
//
// Every call on a GPU shares that GPU's array (each GPU holds its own copy at its own address): the tables are
// rewritten by every call, and calls that overlap in time on one GPU race on them.
#include "host_common.hpp"

#include <mutex>

namespace lpk {

constexpr uint32_t kNoallocMaxTensors = 1u << 14;       // 16384 descriptors (1.1 MiB)
constexpr uint32_t kNoallocMaxTiles   = 1u << 19;       // 524288 tiles = 2^31 elements (8 MiB)

struct NoallocTables {
  Tile      tiles[kNoallocMaxTiles];
  TensorDev tensors[kNoallocMaxTensors];
};

// In host code this name is only a stand-in for the symbol, not a device address: the address on each GPU comes
// from hipGetSymbolAddress (tables_of_current_device), and only that pointer is handed to kernels.
static __device__ __align__(256) unsigned char scratch[sizeof(NoallocTables)];

constexpr int kChunk = 40;                               // descriptors per staging launch: 40 * (72 + 4) B of kernel arguments
struct StageChunk {
  TensorDev t[kChunk];
  uint32_t  first_tile[kChunk];                          // index of each tensor's first tile in the table
};
static_assert(sizeof(StageChunk) <= 3584, "a staging chunk must fit the kernel-argument segment");

// blockIdx.x = tensor within the chunk; the blocks along y share that tensor's tiles.
__global__ void __launch_bounds__(kBlock)
stage_chunk_kernel(StageChunk c, uint32_t base, uint32_t cnt, TensorDev* tensors, Tile* tiles)
{
  const uint32_t j = blockIdx.x;
  if (j >= cnt) return;
  if (blockIdx.y == 0 && threadIdx.x == 0) tensors[base + j] = c.t[j];
  const uint64_t n = c.t[j].n;
  const uint64_t nt = (n + kTileElems - 1) / kTileElems;
  Tile* out = tiles + c.first_tile[j];
  for (uint64_t k = (uint64_t)blockIdx.y * kBlock + threadIdx.x; k < nt; k += (uint64_t)gridDim.y * kBlock) {
    const uint64_t off = k * kTileElems, left = n - off;
    out[k] = Tile{base + j, (uint32_t)(left < (uint64_t)kTileElems ? left : (uint64_t)kTileElems), off};
  }
}

constexpr int kMaxDevices = 64;
struct DeviceSlot { NoallocTables* tables = nullptr; uint32_t n_cu = 0; };
static DeviceSlot g_slot[kMaxDevices];
static std::mutex g_slot_mutex;

// The current device's copy of the array and its CU count, resolved once per device with that device current.
static int tables_of_current_device(DeviceSlot& out)
{
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return LPK_ERR_DEVICE; }
  if (dev < 0 || dev >= kMaxDevices) return LPK_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_slot_mutex);
  if (!g_slot[dev].tables) {
    void* p = nullptr;
    int n_cu = 0;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p ||
        hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0) {
      (void)hipGetLastError();
      return LPK_ERR_DEVICE;
    }
    g_slot[dev].n_cu = (uint32_t)n_cu;
    g_slot[dev].tables = static_cast<NoallocTables*>(p);
  }
  out = g_slot[dev];
  return LPK_OK;
}

}  // namespace lpk

using namespace lpk;

extern "C" int lpk_kahan_sgd_step_noalloc(const lpk_tensor_desc* descs, uint32_t n_tensors,
                                          const int32_t* fl_theta_in, const int32_t* fl_theta_out, const int32_t* fl_grad,
                                          uint32_t lr_q16, uint32_t wd_q16, uint64_t* vmax_out, uint32_t* status, void* stream)
{
  if (!descs || n_tensors == 0 || !fl_theta_in || !fl_theta_out || !fl_grad) return LPK_ERR_INVALID_ARG;
  if (lr_q16 > 65535u || wd_q16 > 65535u) return LPK_ERR_INVALID_ARG;
  if (n_tensors > kNoallocMaxTensors) return LPK_ERR_UNSUPPORTED;

  // first pass: check every descriptor and the size limits before anything is enqueued
  ListFacts facts;
  {
    TensorDev T;
    for (uint32_t t = 0; t < n_tensors; ++t) {
      const int rc = describe_tensor(descs[t], T, facts);
      if (rc != LPK_OK) return rc;
      if (facts.total_tiles > kNoallocMaxTiles) return LPK_ERR_UNSUPPORTED;
    }
  }
  DeviceSlot slot;
  const int rc = tables_of_current_device(slot);
  if (rc != LPK_OK) return rc;
  TensorDev* d_tensors = slot.tables->tensors;           // address arithmetic on the device pointer, no access
  Tile*      d_tiles   = slot.tables->tiles;
  hipStream_t s = static_cast<hipStream_t>(stream);

  // second pass: stage the descriptors chunk by chunk; each launch also writes the tiles of its tensors
  uint32_t next_tile = 0;
  for (uint32_t base = 0; base < n_tensors; base += kChunk) {
    const uint32_t cnt = n_tensors - base < (uint32_t)kChunk ? n_tensors - base : (uint32_t)kChunk;
    StageChunk c{};
    uint64_t most = 0;
    ListFacts ignored;
    for (uint32_t j = 0; j < cnt; ++j) {
      (void)describe_tensor(descs[base + j], c.t[j], ignored);
      c.first_tile[j] = next_tile;
      const uint64_t nt = (descs[base + j].n + kTileElems - 1) / kTileElems;
      next_tile += (uint32_t)nt;
      most = nt > most ? nt : most;
    }
    uint32_t gy = (uint32_t)((most + kBlock - 1) / kBlock);
    gy = gy < 1 ? 1 : (gy > 64 ? 64 : gy);
    hipLaunchKernelGGL(stage_chunk_kernel, dim3(cnt, gy), dim3(kBlock), 0, s, c, base, cnt, d_tensors, d_tiles);
  }
  if (hipGetLastError() != hipSuccess) return LPK_ERR_DEVICE;

  const uint32_t n_tiles = next_tile;
  const uint32_t grid = persistent_grid(n_tiles, slot.n_cu, 2);      // the launch shape of a list with default options
  hipError_t e = launch_kahan_step(d_tensors, d_tiles, n_tiles, n_tensors, grid, 0, fl_theta_in, fl_theta_out, fl_grad,
                                   lr_q16, wd_q16, 0u, facts.any_grad_i8 ? 1u : 0u, vmax_out, status, nullptr, nullptr, s);
  return e == hipSuccess ? LPK_OK : LPK_ERR_DEVICE;
}

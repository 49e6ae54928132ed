// Host layer of liblpk: the C ABI declared in include/lpk.h.  Validates
// arguments, owns the per-list device tables, and enqueues the kernels.
#include "host_common.hpp"

#include <new>
#include <vector>

namespace lpk {
hipError_t launch_select_f32(const TensorDev*, const Tile*, uint32_t n_tiles, uint32_t n_tensors, uint32_t grid,
                             int sel, uint32_t* scratch, uint32_t* arrivals, const int32_t* fl_default, int32_t* fl_out,
                             uint32_t* status, hipStream_t);
hipError_t launch_select_vmax(const TensorDev*, uint32_t n_tensors, int sel, const uint64_t* vmax,
                              const int32_t* fl_theta_in, const int32_t* fl_default, int32_t* fl_out, uint32_t* status,
                              hipStream_t);
hipError_t launch_quantize(const TensorDev*, const Tile*, uint32_t n_tiles, uint32_t grid, int to_theta,
                           const int32_t* fl, uint32_t* status, hipStream_t);
hipError_t launch_select_quantize(const TensorDev*, const Tile*, uint32_t n_tiles, uint32_t n_tensors, uint32_t grid, int to_theta,
                                  const int32_t* fl_guess, int32_t* fl_out, uint32_t* scratch, uint32_t* redo, uint32_t* redo_any,
                                  uint32_t* status, hipStream_t);
hipError_t launch_momentum_step(const TensorDev*, const Tile*, uint32_t n_tiles, uint32_t n_tensors, uint32_t grid,
                                int grad_is_f32, const int32_t* fl_in, const int32_t* fl_out, const int32_t* fl_m_in, const int32_t* fl_m_out,
                                const int32_t* fl_g, uint32_t lr, uint32_t mu, uint32_t wd,
                                uint64_t* vmax, uint64_t* mmax, uint32_t* status, uint64_t* fold_acc, uint32_t* arrivals, hipStream_t);
hipError_t launch_adam_step(const TensorDev*, const Tile*, uint32_t n_tiles, uint32_t n_tensors, uint32_t grid,
                            int grad_is_f32, const int32_t* fl_in, const int32_t* fl_out, const int32_t* fl_m_in, const int32_t* fl_m_out,
                            const int32_t* fl_u_in, const int32_t* fl_u_out, const int32_t* fl_g, AdamHyperDev h,
                            uint64_t* vmax, uint64_t* mmax, uint64_t* umax, uint32_t* status, uint64_t* fold_acc, uint32_t* arrivals,
                            hipStream_t);
}  // namespace lpk

using namespace lpk;

struct lpk_tensor_list {
  uint32_t   n_tensors = 0;
  uint32_t   n_tiles   = 0;
  int        device    = 0;
  uint32_t   grid      = 0;        // blocks of the persistent read-only launch (max-abs) and of the fp32-gradient momentum step
  uint32_t   grid_quant = 0;       // blocks of the quantization launch (4 bytes read : 2 written, out of place)
  uint32_t   grid_step = 0;        // blocks of the plain update launches with lazy stores (read-dominated)
  uint32_t   grid_dense = 0;       // blocks of update launches that write everything (plain with LPK_OPT_STORE_ALL, momentum)
  uint32_t   grid_adam = 0;        // blocks of the ADAM launch
  bool       all_src   = false;    // every non-empty tensor has an fp32 source
  bool       all_mom   = false;    // every non-empty tensor has a velocity buffer
  bool       all_sec   = false;    // ... and a second-moment buffer
  bool       store_all = false;    // LPK_OPT_STORE_ALL: write every result, changed or not
  bool       any_grad_i8 = false;  // some tensor has an int8 gradient array
  uint32_t   n_cu = 0;             // compute units of the list's device
  uint32_t   per_cu[8] = {};       // launch-shape options by lpk_option code, 0 = the built-in default
  TensorDev* d_tensors = nullptr;
  Tile*      d_tiles   = nullptr;
  uint32_t*  d_scratch = nullptr;  // one max word per tensor, zero between calls; then two workgroup counters (max-abs
                                   // scan, update kernels), zero between launches; then lpk_select_quantize's
                                   // "quantize again" flag per tensor and its "any" word
  uint64_t*  d_fold    = nullptr;  // three per-tensor accumulators for the update kernels' maxima, zero between launches
};

// Launch shapes (workgroups of four waves per compute unit) of the persistent kernels; measured on MI355X.
// Long lists are bandwidth-bound: update kernels that write as much as they read stream fastest with ONE workgroup
// (one wave per SIMD) per CU, the read-mostly ones (max-abs, the plain update once its unchanged groups are not
// stored) and ADAM with two; quantization with one on long lists (measured 5 % faster there), two when a wave
// would get fewer than sixteen tiles.
// Short lists of many tensors (fewer than 32 tiles per CU, eight tensors or more -- the parameter set of a small
// network) are latency-bound and their tiles cost unequal time (ragged ends, tiny tensors, mixed widths): there a
// wave should get ONE tile and the hardware should hand out the workgroups, so the grid is as large as the tiles
// need, up to eight workgroups per CU (ResNet-18-sized set: whole step 48 -> 42 us, ResNet-50-sized: 105 -> 83 us).
static void set_grids(lpk_tensor_list* L)
{
  auto grid = [&](uint32_t per_cu) { return persistent_grid(L->n_tiles, L->n_cu, per_cu); };
  const bool short_list = L->n_tensors >= 8 && L->n_tiles < 32u * L->n_cu;
  const uint32_t q_auto = L->n_tiles >= 16u * L->n_cu * kWavesPerBlock ? 1u : 2u;
  auto pick = [&](int opt, uint32_t tuned) { return grid(L->per_cu[opt] ? L->per_cu[opt] : (short_list ? 8u : tuned)); };
  L->grid       = pick(LPK_OPT_SCAN_BLOCKS_PER_CU, 2u);
  L->grid_quant = pick(LPK_OPT_QUANT_BLOCKS_PER_CU, q_auto);
  L->grid_step  = pick(LPK_OPT_STEP_BLOCKS_PER_CU, 2u);
  L->grid_dense = pick(LPK_OPT_DENSE_BLOCKS_PER_CU, 1u);
  L->grid_adam  = pick(LPK_OPT_ADAM_BLOCKS_PER_CU, 2u);
}

// A list belongs to the device that was current when it was made: its tables and the caller's buffers live there.
static bool on_list_device(const lpk_tensor_list* L)
{
  int dev = -1;
  return hipGetDevice(&dev) == hipSuccess && dev == L->device;
}

extern "C" {

int lpk_tensor_list_create(const lpk_tensor_desc* descs, uint32_t n_tensors, lpk_tensor_list** out)
{
  if (out) *out = nullptr;
  if (!descs || !out || n_tensors == 0) return LPK_ERR_INVALID_ARG;

  std::vector<TensorDev> tensors;
  std::vector<Tile> tiles;
  ListFacts facts;
  try {                                              // no exception may cross the C boundary
    tensors.resize(n_tensors);
    for (uint32_t t = 0; t < n_tensors; ++t) {
      const int rc = describe_tensor(descs[t], tensors[t], facts);
      if (rc != LPK_OK) return rc;
    }
    if (facts.total_tiles >= (1ull << 31)) return LPK_ERR_UNSUPPORTED;
    tiles.reserve((size_t)facts.total_tiles);
    for (uint32_t t = 0; t < n_tensors; ++t)
      for (uint64_t off = 0; off < descs[t].n; off += kTileElems) {
        const uint64_t left = descs[t].n - off;
        tiles.push_back(Tile{t, (uint32_t)(left < (uint64_t)kTileElems ? left : (uint64_t)kTileElems), off});
      }
  } catch (...) {
    return LPK_ERR_DEVICE;                           // host memory for the tables could not be had
  }

  lpk_tensor_list* L = new (std::nothrow) lpk_tensor_list;
  if (!L) return LPK_ERR_DEVICE;
  L->n_tensors = n_tensors;
  L->n_tiles = (uint32_t)tiles.size();
  L->all_src = facts.all_src;
  L->all_mom = facts.all_mom;
  L->all_sec = facts.all_sec;
  L->any_grad_i8 = facts.any_grad_i8;

  int n_cu = 0;
  bool ok = hipGetDevice(&L->device) == hipSuccess &&
            hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, L->device) == hipSuccess && n_cu > 0;
  if (ok) {
    L->n_cu = (uint32_t)n_cu;
    set_grids(L);
    ok = hipMalloc((void**)&L->d_tensors, sizeof(TensorDev) * n_tensors) == hipSuccess &&
         hipMalloc((void**)&L->d_scratch, sizeof(uint32_t) * (2 * (size_t)n_tensors + 3)) == hipSuccess &&
         hipMalloc((void**)&L->d_fold, sizeof(uint64_t) * 3 * (size_t)n_tensors) == hipSuccess &&
         (tiles.empty() || hipMalloc((void**)&L->d_tiles, sizeof(Tile) * tiles.size()) == hipSuccess);
  }
  if (ok) {
    ok = hipMemcpy(L->d_tensors, tensors.data(), sizeof(TensorDev) * n_tensors, hipMemcpyHostToDevice) == hipSuccess &&
         hipMemset(L->d_scratch, 0, sizeof(uint32_t) * (2 * (size_t)n_tensors + 3)) == hipSuccess &&
         hipMemset(L->d_fold, 0, sizeof(uint64_t) * 3 * (size_t)n_tensors) == hipSuccess &&
         (tiles.empty() || hipMemcpy(L->d_tiles, tiles.data(), sizeof(Tile) * tiles.size(), hipMemcpyHostToDevice) == hipSuccess) &&
         hipDeviceSynchronize() == hipSuccess;
  }
  if (!ok) {
    (void)hipGetLastError();
    lpk_tensor_list_destroy(L);
    return LPK_ERR_DEVICE;
  }
  *out = L;
  return LPK_OK;
}

int lpk_tensor_list_destroy(lpk_tensor_list* L)
{
  if (!L) return LPK_OK;
  bool ok = true;
  if (L->d_tensors) ok &= hipFree(L->d_tensors) == hipSuccess;
  if (L->d_tiles)   ok &= hipFree(L->d_tiles) == hipSuccess;
  if (L->d_scratch) ok &= hipFree(L->d_scratch) == hipSuccess;
  if (L->d_fold)    ok &= hipFree(L->d_fold) == hipSuccess;
  delete L;
  return ok ? LPK_OK : LPK_ERR_DEVICE;
}

int lpk_tensor_list_set_option(lpk_tensor_list* L, int option, int value)
{
  if (!L) return LPK_ERR_INVALID_ARG;
  if (option == LPK_OPT_STORE_ALL) { L->store_all = value != 0; return LPK_OK; }
  if (option >= LPK_OPT_STEP_BLOCKS_PER_CU && option <= LPK_OPT_QUANT_BLOCKS_PER_CU) {
    if (value < 0 || value > 64) return LPK_ERR_INVALID_ARG;
    L->per_cu[option] = (uint32_t)value;
    set_grids(L);
    return LPK_OK;
  }
  return LPK_ERR_INVALID_ARG;
}

uint32_t lpk_tensor_list_size(const lpk_tensor_list* L) { return L ? L->n_tensors : 0; }
uint64_t lpk_tensor_list_tiles(const lpk_tensor_list* L) { return L ? L->n_tiles : 0; }

int lpk_select_fraclen(lpk_tensor_list* L, int src_kind, int dst_sel,
                       const uint64_t* vmax, const int32_t* fl_theta_in, const int32_t* fl_default,
                       int32_t* fl_out, uint32_t* status, void* stream)
{
  if (!L || !fl_default || !fl_out) return LPK_ERR_INVALID_ARG;
  if (!on_list_device(L)) return LPK_ERR_INVALID_ARG;
  if (dst_sel != LPK_SEL_GRAD && dst_sel != LPK_SEL_THETA && dst_sel != LPK_SEL_MOMENTUM && dst_sel != LPK_SEL_SECOND)
    return LPK_ERR_INVALID_ARG;
  if (dst_sel == LPK_SEL_MOMENTUM && (src_kind != LPK_VMAX_U64 || !L->all_mom)) return LPK_ERR_INVALID_ARG;
  if (dst_sel == LPK_SEL_SECOND && (src_kind != LPK_VMAX_U64 || !L->all_sec)) return LPK_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  if (src_kind == LPK_F32) {
    if (!L->all_src) return LPK_ERR_INVALID_ARG;
    e = launch_select_f32(L->d_tensors, L->d_tiles, L->n_tiles, L->n_tensors, L->grid, dst_sel,
                          L->d_scratch, L->d_scratch + L->n_tensors, fl_default, fl_out, status, s);
  } else if (src_kind == LPK_VMAX_U64) {
    if (!vmax || !fl_theta_in) return LPK_ERR_INVALID_ARG;
    e = launch_select_vmax(L->d_tensors, L->n_tensors, dst_sel, vmax, fl_theta_in, fl_default, fl_out, status, s);
  } else {
    return LPK_ERR_INVALID_ARG;
  }
  return e == hipSuccess ? LPK_OK : LPK_ERR_DEVICE;
}

int lpk_quantize_tensor(lpk_tensor_list* L, int dst_sel, const int32_t* fl, uint32_t* status, void* stream)
{
  if (!L || !fl) return LPK_ERR_INVALID_ARG;
  if (!on_list_device(L)) return LPK_ERR_INVALID_ARG;
  if (dst_sel != LPK_SEL_GRAD && dst_sel != LPK_SEL_THETA) return LPK_ERR_INVALID_ARG;
  if (!L->all_src) return LPK_ERR_INVALID_ARG;
  hipError_t e = launch_quantize(L->d_tensors, L->d_tiles, L->n_tiles, L->grid_quant, dst_sel == LPK_SEL_THETA, fl, status,
                                 static_cast<hipStream_t>(stream));
  return e == hipSuccess ? LPK_OK : LPK_ERR_DEVICE;
}

int lpk_select_quantize(lpk_tensor_list* L, int dst_sel, const int32_t* fl_guess, int32_t* fl_out, uint32_t* status, void* stream)
{
  if (!L || !fl_guess || !fl_out) return LPK_ERR_INVALID_ARG;
  if (!on_list_device(L)) return LPK_ERR_INVALID_ARG;
  if (dst_sel != LPK_SEL_GRAD && dst_sel != LPK_SEL_THETA) return LPK_ERR_INVALID_ARG;
  if (!L->all_src) return LPK_ERR_INVALID_ARG;
  uint32_t* redo = L->d_scratch + L->n_tensors + 2;
  hipError_t e = launch_select_quantize(L->d_tensors, L->d_tiles, L->n_tiles, L->n_tensors, L->grid_quant, dst_sel == LPK_SEL_THETA,
                                        fl_guess, fl_out, L->d_scratch, redo, redo + L->n_tensors, status,
                                        static_cast<hipStream_t>(stream));
  return e == hipSuccess ? LPK_OK : LPK_ERR_DEVICE;
}

int lpk_kahan_sgd_step(lpk_tensor_list* L, const int32_t* fl_theta_in, const int32_t* fl_theta_out, const int32_t* fl_grad,
                       uint32_t lr_q16, uint32_t wd_q16, uint64_t* vmax_out, uint32_t* status, void* stream)
{
  if (!L || !fl_theta_in || !fl_theta_out || !fl_grad) return LPK_ERR_INVALID_ARG;
  if (lr_q16 > 65535u || wd_q16 > 65535u) return LPK_ERR_INVALID_ARG;
  if (!on_list_device(L)) return LPK_ERR_INVALID_ARG;
  hipError_t e = launch_kahan_step(L->d_tensors, L->d_tiles, L->n_tiles, L->n_tensors, L->store_all ? L->grid_dense : L->grid_step, 0, fl_theta_in, fl_theta_out,
                                   fl_grad, lr_q16, wd_q16, L->store_all ? 1u : 0u, L->any_grad_i8 ? 1u : 0u, vmax_out, status,
                                   L->d_fold, L->d_scratch + L->n_tensors + 1, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? LPK_OK : LPK_ERR_DEVICE;
}

int lpk_kahan_sgd_step_f32grad(lpk_tensor_list* L, const int32_t* fl_theta_in, const int32_t* fl_theta_out,
                               const int32_t* fl_grad, uint32_t lr_q16, uint32_t wd_q16, uint64_t* vmax_out,
                               uint32_t* status, void* stream)
{
  if (!L || !fl_theta_in || !fl_theta_out || !fl_grad) return LPK_ERR_INVALID_ARG;
  if (lr_q16 > 65535u || wd_q16 > 65535u) return LPK_ERR_INVALID_ARG;
  if (!on_list_device(L)) return LPK_ERR_INVALID_ARG;
  if (!L->all_src) return LPK_ERR_INVALID_ARG;
  hipError_t e = launch_kahan_step(L->d_tensors, L->d_tiles, L->n_tiles, L->n_tensors, L->store_all ? L->grid_dense : L->grid_step, 1, fl_theta_in, fl_theta_out,
                                   fl_grad, lr_q16, wd_q16, L->store_all ? 1u : 0u, L->any_grad_i8 ? 1u : 0u, vmax_out, status,
                                   L->d_fold, L->d_scratch + L->n_tensors + 1, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? LPK_OK : LPK_ERR_DEVICE;
}

static int momentum_step(lpk_tensor_list* L, int grad_is_f32, const int32_t* fl_theta_in, const int32_t* fl_theta_out,
                         const int32_t* fl_mom_in, const int32_t* fl_mom_out, const int32_t* fl_grad,
                         uint32_t lr_q16, uint32_t mu_q16, uint32_t wd_q16,
                         uint64_t* vmax_out, uint64_t* mmax_out, uint32_t* status, void* stream)
{
  if (!L || !fl_theta_in || !fl_theta_out || !fl_mom_in || !fl_mom_out || !fl_grad) return LPK_ERR_INVALID_ARG;
  if (lr_q16 > 65535u || wd_q16 > 65535u || mu_q16 > 65535u) return LPK_ERR_INVALID_ARG;
  if (!on_list_device(L)) return LPK_ERR_INVALID_ARG;
  if (!L->all_mom || (grad_is_f32 && !L->all_src)) return LPK_ERR_INVALID_ARG;
  // fed from fp32 gradients the stream reads 7 bytes per 3 written and runs slightly faster with two workgroups per CU
  hipError_t e = launch_momentum_step(L->d_tensors, L->d_tiles, L->n_tiles, L->n_tensors, grad_is_f32 ? L->grid : L->grid_dense, grad_is_f32,
                                      fl_theta_in, fl_theta_out, fl_mom_in, fl_mom_out, fl_grad, lr_q16, mu_q16, wd_q16,
                                      vmax_out, mmax_out, status, L->d_fold, L->d_scratch + L->n_tensors + 1,
                                      static_cast<hipStream_t>(stream));
  return e == hipSuccess ? LPK_OK : LPK_ERR_DEVICE;
}

int lpk_momentum_sgd_step(lpk_tensor_list* L, const int32_t* fl_theta_in, const int32_t* fl_theta_out,
                          const int32_t* fl_mom_in, const int32_t* fl_mom_out, const int32_t* fl_grad,
                          uint32_t lr_q16, uint32_t mu_q16, uint32_t wd_q16,
                          uint64_t* vmax_out, uint64_t* mmax_out, uint32_t* status, void* stream)
{
  return momentum_step(L, 0, fl_theta_in, fl_theta_out, fl_mom_in, fl_mom_out, fl_grad, lr_q16, mu_q16, wd_q16,
                       vmax_out, mmax_out, status, stream);
}

int lpk_momentum_sgd_step_f32grad(lpk_tensor_list* L, const int32_t* fl_theta_in, const int32_t* fl_theta_out,
                                  const int32_t* fl_mom_in, const int32_t* fl_mom_out, const int32_t* fl_grad,
                                  uint32_t lr_q16, uint32_t mu_q16, uint32_t wd_q16,
                                  uint64_t* vmax_out, uint64_t* mmax_out, uint32_t* status, void* stream)
{
  return momentum_step(L, 1, fl_theta_in, fl_theta_out, fl_mom_in, fl_mom_out, fl_grad, lr_q16, mu_q16, wd_q16,
                       vmax_out, mmax_out, status, stream);
}

static int adam_step(lpk_tensor_list* L, int grad_is_f32, const int32_t* fl_theta_in, const int32_t* fl_theta_out,
                     const int32_t* fl_mom_in, const int32_t* fl_mom_out, const int32_t* fl_sec_in, const int32_t* fl_sec_out,
                     const int32_t* fl_grad, const lpk_adam_hyper* hyper,
                     uint64_t* vmax_out, uint64_t* mmax_out, uint64_t* umax_out, uint32_t* status, void* stream)
{
  if (!L || !fl_theta_in || !fl_theta_out || !fl_mom_in || !fl_mom_out || !fl_sec_in || !fl_sec_out || !fl_grad || !hyper)
    return LPK_ERR_INVALID_ARG;
  if (hyper->lr_q16 > 65535u || hyper->beta1_q16 > 65535u || hyper->beta2_q16 > 65535u || hyper->eps_q16 > 65535u ||
      hyper->lr_exp > 48u || hyper->eps_exp > 48u) return LPK_ERR_INVALID_ARG;
  if (!on_list_device(L)) return LPK_ERR_INVALID_ARG;
  if (!L->all_mom || !L->all_sec || (grad_is_f32 && !L->all_src)) return LPK_ERR_INVALID_ARG;
  const AdamHyperDev h{hyper->lr_q16, hyper->lr_exp, hyper->beta1_q16, hyper->beta2_q16, hyper->eps_q16, hyper->eps_exp};
  hipError_t e = launch_adam_step(L->d_tensors, L->d_tiles, L->n_tiles, L->n_tensors, L->grid_adam, grad_is_f32,
                                  fl_theta_in, fl_theta_out, fl_mom_in, fl_mom_out, fl_sec_in, fl_sec_out, fl_grad, h,
                                  vmax_out, mmax_out, umax_out, status, L->d_fold, L->d_scratch + L->n_tensors + 1,
                                  static_cast<hipStream_t>(stream));
  return e == hipSuccess ? LPK_OK : LPK_ERR_DEVICE;
}

int lpk_adam_step(lpk_tensor_list* L, const int32_t* fl_theta_in, const int32_t* fl_theta_out,
                  const int32_t* fl_mom_in, const int32_t* fl_mom_out, const int32_t* fl_sec_in, const int32_t* fl_sec_out,
                  const int32_t* fl_grad, const lpk_adam_hyper* hyper,
                  uint64_t* vmax_out, uint64_t* mmax_out, uint64_t* umax_out, uint32_t* status, void* stream)
{
  return adam_step(L, 0, fl_theta_in, fl_theta_out, fl_mom_in, fl_mom_out, fl_sec_in, fl_sec_out, fl_grad, hyper,
                   vmax_out, mmax_out, umax_out, status, stream);
}

int lpk_adam_step_f32grad(lpk_tensor_list* L, const int32_t* fl_theta_in, const int32_t* fl_theta_out,
                          const int32_t* fl_mom_in, const int32_t* fl_mom_out, const int32_t* fl_sec_in, const int32_t* fl_sec_out,
                          const int32_t* fl_grad, const lpk_adam_hyper* hyper,
                          uint64_t* vmax_out, uint64_t* mmax_out, uint64_t* umax_out, uint32_t* status, void* stream)
{
  return adam_step(L, 1, fl_theta_in, fl_theta_out, fl_mom_in, fl_mom_out, fl_sec_in, fl_sec_out, fl_grad, hyper,
                   vmax_out, mmax_out, umax_out, status, stream);
}

const char* lpk_error_string(int code)
{
  switch (code) {
    case LPK_OK:              return "ok";
    case LPK_ERR_INVALID_ARG: return "invalid argument";
    case LPK_ERR_UNSUPPORTED: return "unsupported request";
    case LPK_ERR_DEVICE:      return "HIP runtime failure";
    default:                  return "unknown lpk status code";
  }
}

int lpk_classifier_min_bits(uint32_t n_classes, uint32_t alpha_q16)
{
  if (n_classes < 2 || alpha_q16 == 0 || alpha_q16 > 65535u) return LPK_ERR_INVALID_ARG;
  // 2^(BW-1) >= (n-1) / alpha  <=>  alpha_q16 << (BW-1) >= (n-1) << 16; the left side grows past any 48-bit right side
  const uint64_t need = (uint64_t)(n_classes - 1) << 16;
  int bw = 2;
  while (((uint64_t)alpha_q16 << (bw - 1)) < need) ++bw;
  return bw;
}

int lpk_version(void) { return 300; }      // 0.3.0: lpk_select_quantize

}  // extern "C"

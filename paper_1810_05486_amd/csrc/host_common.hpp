// Host-side helpers shared by the entry points of liblpk: turning one caller descriptor into the form the kernels
// read, with the argument checks every entry point applies.
#pragma once
#include "../../include/lpk.h"
#include "lpk_device.hpp"

namespace lpk {

inline int dtype_bits(uint8_t dt) { return dt == LPK_I8 ? 8 : (dt == LPK_I16 ? 16 : 0); }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// What a whole list has in common, gathered while its descriptors are checked.
struct ListFacts {
  bool     all_src = true;       // every non-empty tensor has an fp32 source
  bool     all_mom = true;       // ... a velocity / first-moment buffer
  bool     all_sec = true;       // ... a second-moment buffer
  bool     any_grad_i8 = false;  // some tensor has an int8 gradient array
  uint64_t total_tiles = 0;
};

// Check one descriptor (dtype codes, comp shift, NULL and alignment rules of lpk_tensor_desc) and fill the
// kernels' view of it.  Returns LPK_OK or LPK_ERR_INVALID_ARG.
inline int describe_tensor(const lpk_tensor_desc& D, TensorDev& T, ListFacts& f)
{
  const int wt = dtype_bits(D.theta_dtype), wg = dtype_bits(D.grad_dtype);
  const int wc = D.comp ? dtype_bits(D.comp_dtype) : 0;
  if (!wt || !wg || (D.comp && !wc)) return LPK_ERR_INVALID_ARG;
  int d = 0;
  if (D.comp) {
    d = D.comp_shift == LPK_COMP_SHIFT_DEFAULT ? wc - 1 : (int)D.comp_shift;
    if (d > kDMax) return LPK_ERR_INVALID_ARG;
  }
  if (D.n && (!D.theta || !D.grad)) return LPK_ERR_INVALID_ARG;
  if (!aligned(D.theta, wt / 8) || !aligned(D.grad, wg / 8) || (D.comp && !aligned(D.comp, wc / 8)) ||
      !aligned(D.src_f32, 4)) return LPK_ERR_INVALID_ARG;
  if (D.n && !D.src_f32) f.all_src = false;
  if (D.n && wg == 8) f.any_grad_i8 = true;
  const int wm = D.momentum ? dtype_bits(D.momentum_dtype) : 0;
  if (D.momentum && (!wm || !aligned(D.momentum, wm / 8))) return LPK_ERR_INVALID_ARG;
  if (D.n && !D.momentum) f.all_mom = false;
  const int wu = D.second ? dtype_bits(D.second_dtype) : 0;
  if (D.second && (!wu || !aligned(D.second, wu / 8))) return LPK_ERR_INVALID_ARG;
  if (D.n && !D.second) f.all_sec = false;

  T = TensorDev{};
  T.theta = D.theta; T.comp = D.comp; T.grad = const_cast<void*>(D.grad); T.src = D.src_f32; T.n = D.n;
  T.wt = (uint8_t)wt; T.wc = (uint8_t)wc; T.wg = (uint8_t)wg; T.d = (uint8_t)d;
  T.vec_step      = aligned(D.theta, 16) && aligned(D.grad, 16) && D.comp && aligned(D.comp, 16);
  T.vec_src_grad  = D.src_f32 && aligned(D.src_f32, 16) && aligned(D.grad, 16);
  T.vec_src_theta = D.src_f32 && aligned(D.src_f32, 16) && aligned(D.theta, 16);
  T.mom = D.momentum; T.wm = (uint8_t)wm;
  T.vec_mom = T.vec_step && D.momentum && aligned(D.momentum, 16);
  T.sec = D.second; T.wu = (uint8_t)wu;
  T.vec_adam = T.vec_mom && D.second && aligned(D.second, 16);
  f.total_tiles += (D.n + kTileElems - 1) / kTileElems;
  return LPK_OK;
}

// Blocks of a persistent launch: `per_cu` workgroups per compute unit, never more than the tiles need.
inline uint32_t persistent_grid(uint32_t n_tiles, uint32_t n_cu, uint32_t per_cu)
{
  const uint32_t need = (n_tiles + kWavesPerBlock - 1) / kWavesPerBlock;
  uint32_t g = n_cu * per_cu;
  if (g > need) g = need;
  return g ? g : 1u;
}

hipError_t launch_kahan_step(const TensorDev*, const Tile*, uint32_t n_tiles, uint32_t n_tensors, uint32_t grid,
                             int grad_is_f32, const int32_t*, const int32_t*, const int32_t*, uint32_t lr, uint32_t wd,
                             uint32_t store_all, uint32_t with_i8, uint64_t* vmax, uint32_t* status,
                             uint64_t* fold_acc, uint32_t* arrivals, hipStream_t);

}  // namespace lpk

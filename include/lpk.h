/*
 * lpk.h -- C ABI of the MI355X (gfx950) library for the low-precision SGD
 * parameter update with Kahan summation ("lazy update") over dynamic
 * fixed-point (DFX) parameters.
 *
 * Paper: "Training Deep Neural Network in Limited Precision" (Park et al.).
 *   Section 2 + Algorithm 1 : the update (an extra accumulation parameter
 *                             carries the part of each step that the parameter's
 *                             precision cannot hold).
 *   Section 2, Figure 1     : parameter, gradient and accumulator on one
 *                             decimal-point axis; effective width m+n-2-k.
 *   Section 1               : 8/16-bit dynamic fixed point, uniform linear
 *                             quantization, no stochastic rounding.
 *   Section 6               : a tensor's exponent is chosen from its maximum.
 *
 * Number format.  DFX(W, fl): a two's-complement integer q of W in {8, 16}
 * bits standing for q * 2^-fl; fl ("fractional length") is shared by a whole
 * tensor.  qmax = 2^(W-1)-1, qmin = -2^(W-1).  RNE = round to nearest, ties
 * to even; sat_W clamps to [qmin, qmax].
 *
 * The compensation tensor `comp` holds c = -acc of Algorithm 1, on the grid
 * fl_theta + d, where d (`comp_shift`) is the distance between the two
 * decimal points; d = bits(comp) - 1 means no overlapping bit (k = 0).
 *
 * Conventions for every call.
 *   - Return value: LPK_OK (0) or a negative lpk_status_code.  Argument errors
 *     are detected on the host before anything is launched.
 *   - Pointers marked "device" are HIP device pointers; everything else is
 *     host memory.  `stream` is a hipStream_t passed as void* (NULL = the
 *     default stream).  Work is only enqueued: no call synchronizes, and the
 *     three hot calls allocate nothing.
 *   - The caller owns every data buffer, fraclen / vmax / status array and the
 *     stream.  The library owns only what lpk_tensor_list_create allocates.
 *   - Data-dependent conditions are not errors: their bits are OR-ed into
 *     status[0] (device uint32, may be NULL) -- see LPK_STATUS_*.
 *   - Domain: fraclens in [-64, 64]; 0 <= d <= 24; |fl_out - fl_in| <= 15;
 *     lr_q16, wd_q16 <= 65535.  A tensor whose device-side fraclens fall
 *     outside it is skipped untouched and LPK_STATUS_DOMAIN is raised.
 *   - Calls on one list that overlap in time (different streams) race on the
 *     list's reduction scratch; serialize them.
 *   - One device per list: a list belongs to the device that was current in
 *     lpk_tensor_list_create, its buffers live there, and every later call on
 *     it must be made with that device current (else INVALID_ARG).
 */
#ifndef LPK_H
#define LPK_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LPK_OK              =  0,
  LPK_ERR_INVALID_ARG = -1,  /* NULL where forbidden, bad dtype / selector code, n_tensors == 0,
                                misaligned pointer, lr/wd above 65535; nothing was launched   */
  LPK_ERR_UNSUPPORTED = -2,  /* a well-formed request this build does not implement          */
  LPK_ERR_DEVICE      = -3   /* a HIP runtime call failed (allocation, copy, launch), or host memory ran out */
} lpk_status_code;

typedef enum { LPK_I8 = 1, LPK_I16 = 2, LPK_F32 = 4, LPK_VMAX_U64 = 8 } lpk_dtype;

/* which member of the descriptor a call reads its width from / writes to */
typedef enum { LPK_SEL_GRAD = 0, LPK_SEL_THETA = 1, LPK_SEL_MOMENTUM = 2, LPK_SEL_SECOND = 3 } lpk_selector;

/* bits of the device status word */
#define LPK_STATUS_NONFINITE 1u  /* a NaN or Inf was met in fp32 input                               */
#define LPK_STATUS_DOMAIN    2u  /* a fraclen or shift outside the domain; that tensor was skipped   */

#define LPK_COMP_SHIFT_DEFAULT 0xFFu

/* One tensor of the parameter set.  Host array, copied at list creation.
 * Element pointers must be aligned to their element size; when theta, comp,
 * grad (and src_f32, and the optimizer states) are all 16-byte aligned the
 * tensor takes the vector path (more than ten times faster than the
 * element-by-element one).  The vector path covers: comp as wide as theta, or
 * int8 theta with an int16 comp; 16-bit gradients
 * with any of these; int8 gradients (Section 4's 8-bit training) next to an
 * int8 theta; for ADAM 16-bit moments and gradients.  Anything else is
 * computed element by element, with the same results.
 * Buffers of one tensor and of different tensors must not overlap. */
typedef struct {
  void*       theta;       /* device; DFX ints, updated in place; destination of quantize(LPK_SEL_THETA) */
  void*       comp;        /* device; DFX ints, updated in place; NULL = plain SGD without the accumulator */
  const void* grad;        /* device; DFX ints; destination of quantize(LPK_SEL_GRAD)                      */
  const void* src_f32;     /* device; fp32 source of select_fraclen(LPK_F32) / quantize; may be NULL       */
  uint64_t    n;           /* elements (0 allowed: the tensor is a no-op)                                  */
  uint8_t     theta_dtype; /* LPK_I8 or LPK_I16 */
  uint8_t     comp_dtype;  /* LPK_I8 or LPK_I16 (ignored when comp == NULL) */
  uint8_t     grad_dtype;  /* LPK_I8 or LPK_I16 */
  uint8_t     comp_shift;  /* d = fl_comp - fl_theta, 0..24; LPK_COMP_SHIFT_DEFAULT = bits(comp_dtype) - 1 */
  uint8_t     momentum_dtype; /* LPK_I8 or LPK_I16 (ignored when momentum == NULL) */
  uint8_t     second_dtype;   /* LPK_I8 or LPK_I16 (ignored when second == NULL) */
  uint8_t     reserved[2];    /* set to 0 */
  void*       momentum;    /* device; DFX ints, updated in place; may be NULL.  The velocity of
                              lpk_momentum_sgd_step, the first moment of lpk_adam_step                      */
  void*       second;      /* device; DFX ints >= 0, second moment of lpk_adam_step, updated in place; may be NULL */
} lpk_tensor_desc;

typedef struct lpk_tensor_list lpk_tensor_list;   /* opaque */

/* Build the multi-tensor list: validates the descriptors, cuts every tensor
 * into tiles, and uploads the descriptor table, the tile table and the
 * reduction scratch to the CURRENT device.  Allocates device memory and
 * synchronizes once.  *out is NULL on failure.
 * Errors: INVALID_ARG (NULL descs/out, n_tensors == 0, bad dtype, d > 24,
 * NULL theta/grad with n > 0, pointer not aligned to its element size),
 * DEVICE. */
int lpk_tensor_list_create(const lpk_tensor_desc* descs, uint32_t n_tensors, lpk_tensor_list** out);

/* Free what _create allocated.  NULL is accepted.  The caller must have
 * synchronized every stream that still uses the list. */
int lpk_tensor_list_destroy(lpk_tensor_list* list);

/* Per-list options; each takes effect for calls enqueued afterwards.
 *   LPK_OPT_STORE_ALL (default 0): the plain update kernels normally do not issue the store of a 16-byte group of
 *     theta or comp whose new value equals the one loaded (in the lazy update most parameters do not move in a step,
 *     so this saves most of the write traffic); with value 1 every result is written.  The results in memory are the
 *     same either way.
 *   LPK_OPT_*_BLOCKS_PER_CU: launch shape of one family of kernels, in workgroups (of four wavefronts) per compute
 *     unit, 1..64; 0 restores the built-in choice.  STEP: the plain update with lazy stores (built-in 2); DENSE: the
 *     plain update with LPK_OPT_STORE_ALL and the momentum update (1); ADAM: the ADAM update (2); SCAN: the max-abs
 *     scan of lpk_select_fraclen and the fp32-gradient momentum update (2); QUANT: lpk_quantize_tensor and lpk_select_quantize (1 on long
 *     lists, 2 on short ones); every family 8 on short lists of many tensors (at least 8 tensors, fewer than 32
 *     tiles of 4096 elements per compute unit).  The grid never exceeds what the tiles need.  Results do not depend
 *     on the launch shape; these exist for tuning on other parts.
 * Errors: INVALID_ARG (NULL list, unknown option, value out of range). */
typedef enum {
  LPK_OPT_STORE_ALL = 1,
  LPK_OPT_STEP_BLOCKS_PER_CU = 2, LPK_OPT_DENSE_BLOCKS_PER_CU = 3, LPK_OPT_ADAM_BLOCKS_PER_CU = 4,
  LPK_OPT_SCAN_BLOCKS_PER_CU = 5, LPK_OPT_QUANT_BLOCKS_PER_CU = 6
} lpk_option;
int lpk_tensor_list_set_option(lpk_tensor_list* list, int option, int value);

/* Number of tensors / of tiles in a list (host-side facts, no device access); 0 for NULL. */
uint32_t lpk_tensor_list_size(const lpk_tensor_list* list);
uint64_t lpk_tensor_list_tiles(const lpk_tensor_list* list);

/*
 * Fractional length per tensor from a max-abs reduction (Section 6: the
 * exponent follows the scanned maximum; Section 1: dynamic fixed point).
 *
 *   fl*(M, W) = the largest fl with RNE(M * 2^fl) <= 2^(W-1) - 1, clamped to [-64, 64]:
 *   the finest grid on which the tensor's own maximum does not saturate.
 *
 * W = bits of desc.grad_dtype (dst_sel == LPK_SEL_GRAD), desc.theta_dtype
 * (LPK_SEL_THETA), desc.momentum_dtype (LPK_SEL_MOMENTUM) or desc.second_dtype
 * (LPK_SEL_SECOND); the last two with LPK_VMAX_U64 only.
 *
 * src_kind == LPK_F32: M = max_i |desc.src_f32[i]| (src_f32 must be non-NULL
 *   for every tensor with n > 0).  M == 0 (or n == 0) -> fl_default[t].  Any
 *   NaN/Inf in the tensor -> -64 and LPK_STATUS_NONFINITE.  vmax and
 *   fl_theta_in are ignored (may be NULL).
 *
 * src_kind == LPK_VMAX_U64: M = vmax[t] * 2^-(fl_theta_in[t] + d_t): the
 *   running maximum that lpk_kahan_sgd_step wrote when it was called with
 *   fl_theta_in (d_t = the tensor's comp shift, 0 without comp).  vmax[t] == 0
 *   -> fl_default[t].  The result is additionally clamped to
 *   fl_default[t] +- 15, so that it can be handed to the next step as
 *   fl_theta_out when fl_default is that step's fl_theta_in.
 *   With dst_sel == LPK_SEL_MOMENTUM the maximum is the mmax of
 *   lpk_momentum_sgd_step and `fl_theta_in` is the fl_mom_out array that step
 *   was called with: M = vmax[t] * 2^-fl_theta_in[t].  The same holds for the mmax
 *   (LPK_SEL_MOMENTUM, fl_mom_out) and the umax (LPK_SEL_SECOND, fl_sec_out) of lpk_adam_step.
 *
 * vmax (uint64), fl_theta_in, fl_default, fl_out (int32): device arrays of
 * n_tensors entries.  fl_out is written for every tensor.
 */
int lpk_select_fraclen(lpk_tensor_list* list, int src_kind, int dst_sel,
                       const uint64_t* vmax, const int32_t* fl_theta_in, const int32_t* fl_default,
                       int32_t* fl_out, uint32_t* status, void* stream);

/*
 * Uniform linear quantization, no stochastic rounding (Section 1):
 *   dst[i] = sat_W( RNE( src_f32[i] * 2^fl[t] ) )
 * dst = desc.grad (dst_sel == LPK_SEL_GRAD; written although declared const in
 * the descriptor, because the update only reads it) or desc.theta
 * (LPK_SEL_THETA); W from the matching dtype.  NaN -> 0, +-Inf -> qmax/qmin,
 * both raise LPK_STATUS_NONFINITE.  fl[t] outside [-64, 64]: tensor skipped,
 * LPK_STATUS_DOMAIN.  fl: device int32[n_tensors].
 */
int lpk_quantize_tensor(lpk_tensor_list* list, int dst_sel, const int32_t* fl,
                        uint32_t* status, void* stream);

/*
 * lpk_select_fraclen(LPK_F32, dst_sel) followed by lpk_quantize_tensor(dst_sel), with ONE read of the fp32 data
 * where the caller's guess holds (Section 6: the exponent follows the scanned maximum; it also mentions the
 * history of maxima, and from one training step to the next a tensor's exponent rarely changes).
 * fl_guess[t] is the fraclen the caller expects for tensor t -- normally last step's -- and, as fl_default does in
 * lpk_select_fraclen, the value an empty or all-zero tensor keeps.  The pass quantizes every tensor with its guess
 * while it scans for the maximum; the true fraclen from the maximum goes to fl_out[t]; a tensor whose guess was
 * wrong (or outside [-64, 64]) is quantized again with the true one.  Tensors of at most 4096 elements never need
 * that: one wavefront finds the maximum first.  dst, fl_out and the status word end up exactly as after the two
 * calls with fl_default = fl_guess; only the time differs (a wrong guess costs one more pass over that tensor).
 * fl_guess, fl_out: device int32[n_tensors]; they may be the same array.  Every non-empty tensor needs src_f32.
 * Errors: INVALID_ARG (NULL argument, bad dst_sel, a tensor without src_f32, wrong device), DEVICE.
 */
int lpk_select_quantize(lpk_tensor_list* list, int dst_sel, const int32_t* fl_guess, int32_t* fl_out,
                        uint32_t* status, void* stream);

/*
 * One lazy-update step over every tensor of the list in a single fused launch
 * (Algorithm 1; eq. 1 when comp == NULL).  Per tensor t and element i, with
 * F = fl_theta_in[t] + d the working grid (units: LSBs of c) and
 * cap(x) = clamp(x, -2^40, 2^40):
 *
 *   s  = cap(RNE(-lr_q16 * g * 2^-(fl_grad[t] + 16 - F)))               step, on c's grid
 *      + cap(RNE(-lr_q16 * wd_q16 * theta * 2^-(32 - d)))               if wd_q16 != 0
 *   v  = theta * 2^d + c + s                                            compensated sum, kept wide
 *   theta' = sat( RNE( v * 2^(fl_theta_out[t] - F) ) )                  the part theta can hold
 *   c'     = sat( RNE( (v * 2^-F - theta' * 2^-fl_theta_out[t]) * 2^(fl_theta_out[t] + d) ) )   the rest
 *   vmax_out[t] = max_i |v_i|                                           (on grid F)
 *
 * theta leaves the call on grid fl_theta_out[t], comp on fl_theta_out[t] + d.
 * fl_theta_in, fl_theta_out (may be the same array), fl_grad: device
 * int32[n_tensors].  vmax_out: device uint64[n_tensors] or NULL; it is
 * cleared and rewritten by every call.  lr_q16, wd_q16: unsigned Q0.16
 * (value / 65536), at most 65535; wd_q16 == 0 switches decay off.
 */
int lpk_kahan_sgd_step(lpk_tensor_list* list,
                       const int32_t* fl_theta_in, const int32_t* fl_theta_out, const int32_t* fl_grad,
                       uint32_t lr_q16, uint32_t wd_q16,
                       uint64_t* vmax_out, uint32_t* status, void* stream);

/*
 * The same update fed from the fp32 gradients: exactly lpk_quantize_tensor(LPK_SEL_GRAD, fl_grad) followed by
 * lpk_kahan_sgd_step, in ONE pass that reads desc.src_f32, quantizes each gradient in registers
 * (sat_W(RNE(x * 2^fl_grad[t])), W = bits(grad_dtype); NaN -> 0, +-Inf -> rails, LPK_STATUS_NONFINITE) and never
 * touches desc.grad -- the int16 round trip through HBM (2 B written + 2 B read per element) disappears.
 * Results (theta, comp, vmax, status) are bit-identical to the two-call sequence.  Every non-empty tensor
 * needs src_f32 (else INVALID_ARG); fl_grad normally comes from lpk_select_fraclen(LPK_F32, LPK_SEL_GRAD).
 */
int lpk_kahan_sgd_step_f32grad(lpk_tensor_list* list,
                               const int32_t* fl_theta_in, const int32_t* fl_theta_out, const int32_t* fl_grad,
                               uint32_t lr_q16, uint32_t wd_q16,
                               uint64_t* vmax_out, uint32_t* status, void* stream);

/*
 * lpk_kahan_sgd_step for callers that cannot allocate device memory: code running under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  It needs no lpk_tensor_list: it takes the host array of
 * descriptors itself and keeps the tables that lpk_tensor_list_create would allocate in a fixed device array inside
 * the library (9.1 MiB, held by every GPU the library runs on until the process ends).  The call allocates nothing,
 * frees nothing and does not synchronize; the descriptors reach the device as kernel arguments, so `descs` may be
 * reused as soon as the call returns.  Results (theta, comp, vmax_out, status) are bit-identical to
 * lpk_tensor_list_create + lpk_kahan_sgd_step with default options on the same descriptors.
 * Limits: n_tensors <= 16384 and at most 524288 tiles, a tile being 4096 elements of one tensor, counted per
 * tensor as ceil(n / 4096) (so up to 2^31 elements in one tensor); beyond them LPK_ERR_UNSUPPORTED, nothing launched.
 * Every call on a GPU rewrites that GPU's array: calls that overlap in time on one GPU (different streams, or
 * threads) race on it and must be serialized by the caller; calls on one stream are ordered by the stream.
 * Other arguments and errors as lpk_kahan_sgd_step (INVALID_ARG also for what lpk_tensor_list_create rejects).
 */
int lpk_kahan_sgd_step_noalloc(const lpk_tensor_desc* descs /* host */, uint32_t n_tensors,
                               const int32_t* fl_theta_in, const int32_t* fl_theta_out, const int32_t* fl_grad,
                               uint32_t lr_q16, uint32_t wd_q16,
                               uint64_t* vmax_out, uint32_t* status, void* stream);

/*
 * Momentum SGD with the lazy update inside (Section 4: the momentum optimizer, mu = 0.9, with Algorithm 1
 * implemented in the optimizer; INT8 or INT16 velocity).  Heavy-ball form with the learning rate inside
 * the velocity:  m <- mu*m - lr*(g + wd*theta);  theta <- theta + m  through Algorithm 1.
 * desc.momentum (non-NULL for every tensor with n > 0) holds m in DFX(bits(momentum_dtype), fl_mom).
 * Per element, with G = fl_mom_out[t] + 16 (16 guard bits below the velocity's LSB) and F, cap as above:
 *
 *   w  = RNE(mu_q16 * m * 2^-(fl_mom_in[t] - fl_mom_out[t]))                 (exact unless the grid coarsens)
 *      + cap(RNE(-lr_q16 * g * 2^-(fl_grad[t] - fl_mom_out[t])))
 *      + cap(RNE(-lr_q16 * wd_q16 * theta * 2^-(fl_theta_in[t] + 16 - fl_mom_out[t])))     if wd_q16 != 0
 *   mq = RNE(w * 2^-16);  m' = sat(mq)                                        stored on grid fl_mom_out[t]
 *   s  = cap(RNE(m' * 2^-(fl_mom_out[t] - F)))
 *   v, theta', c', vmax_out exactly as in lpk_kahan_sgd_step with this s;  mmax_out[t] = max_i |mq_i|
 *
 * fl_mom_in / fl_mom_out: device int32[n_tensors], in [-64, 64], |difference| <= 15.  mu_q16 <= 65535.
 * mmax_out: device uint64[n_tensors] or NULL, cleared and rewritten by the call; feed it to
 * lpk_select_fraclen(LPK_VMAX_U64, LPK_SEL_MOMENTUM) to re-select the velocity's fraclen.
 * Errors: as lpk_kahan_sgd_step, plus INVALID_ARG when a non-empty tensor has no momentum buffer.
 */
int lpk_momentum_sgd_step(lpk_tensor_list* list,
                          const int32_t* fl_theta_in, const int32_t* fl_theta_out,
                          const int32_t* fl_mom_in, const int32_t* fl_mom_out, const int32_t* fl_grad,
                          uint32_t lr_q16, uint32_t mu_q16, uint32_t wd_q16,
                          uint64_t* vmax_out, uint64_t* mmax_out, uint32_t* status, void* stream);

/*
 * The same momentum step fed from the fp32 gradients (Sections 1, 2, 4): exactly
 * lpk_quantize_tensor(LPK_SEL_GRAD, fl_grad) followed by lpk_momentum_sgd_step, in ONE pass that reads desc.src_f32,
 * quantizes each gradient in registers as lpk_kahan_sgd_step_f32grad does, and never touches desc.grad.  Results
 * (theta, comp, momentum, vmax, mmax, status) are bit-identical to the two-call sequence.  Every non-empty tensor
 * needs src_f32 and a momentum buffer (else INVALID_ARG).
 */
int lpk_momentum_sgd_step_f32grad(lpk_tensor_list* list,
                                  const int32_t* fl_theta_in, const int32_t* fl_theta_out,
                                  const int32_t* fl_mom_in, const int32_t* fl_mom_out, const int32_t* fl_grad,
                                  uint32_t lr_q16, uint32_t mu_q16, uint32_t wd_q16,
                                  uint64_t* vmax_out, uint64_t* mmax_out, uint32_t* status, void* stream);

/*
 * ADAM with the lazy update inside (Section 4: the ADAM optimizer in INT16 -- 16 bits because of beta2 --
 * with Algorithm 1 implemented in the optimizer; the paper names only the hyper-parameters).  Textbook rule
 *   m <- beta1 m + (1 - beta1) g;  u <- beta2 u + (1 - beta2) g^2;  theta <- theta - lr_t m / (sqrt(u) + eps)
 * with the bias corrections folded into lr_t = lr sqrt(1 - beta2^t) / (1 - beta1^t) by the caller, and the step
 * handed to Algorithm 1's accumulator.  desc.momentum holds m in DFX(bits(momentum_dtype), fl_mom), desc.second
 * holds u >= 0 in DFX(bits(second_dtype), fl_sec); both non-NULL for every tensor with n > 0.
 * Per element (every RNE as if in unbounded integers; cap = clamp to +-2^40; F = fl_theta_in[t] + d):
 *
 *   wM = RNE(beta1_q16 * m * 2^-(fl_mom_in[t] - fl_mom_out[t])) + cap(RNE((65536 - beta1_q16) * g * 2^-(fl_grad[t] - fl_mom_out[t])))
 *   mq = RNE(wM * 2^-16);  m' = sat(mq);  mmax_out[t] = max_i |mq_i|
 *   wU = RNE(beta2_q16 * u * 2^-(fl_sec_in[t] - fl_sec_out[t])) + cap(RNE((65536 - beta2_q16) * g^2 * 2^-(2 fl_grad[t] - fl_sec_out[t])))
 *   uq = RNE(wU * 2^-16);  u' = clamp(uq, 0, qmax);  umax_out[t] = max_i max(uq_i, 0)
 *   rt = floor(sqrt(u' * 2^(24 + p))),  p = fl_sec_out[t] mod 2 in {0, 1}: the root on grid R = (fl_sec_out[t] + 24 + p) / 2
 *   den = max(rt + min(RNE(eps_q16 * 2^-(16 + eps_exp - R)), 2^30), 1)
 *   s  = cap(RNE(-lr_q16 * m' * 2^e / den)),  e = F + R - 16 - lr_exp - fl_mom_out[t]
 *   v, theta', c', vmax_out exactly as in lpk_kahan_sgd_step with this s
 *
 * lr_t = lr_q16 * 2^-(16 + lr_exp), eps = eps_q16 * 2^-(16 + eps_exp): 16-bit mantissas, exponents 0..48.
 * Domain, beyond that of lpk_kahan_sgd_step: the four moment fraclens in [-64, 64], each pair at most 15
 * apart, and e <= 20; outside it the tensor is skipped and LPK_STATUS_DOMAIN raised.
 * mmax_out, umax_out: device uint64[n_tensors] or NULL, cleared and rewritten by the call; feed them to
 * lpk_select_fraclen(LPK_VMAX_U64, LPK_SEL_MOMENTUM / LPK_SEL_SECOND) to re-select the moments' fraclens.
 * Errors: INVALID_ARG (NULL list / fraclen array / hyper, a mantissa above 65535, an exponent above 48, a
 * non-empty tensor without momentum or second buffer), DEVICE.
 */
typedef struct {
  uint32_t lr_q16, lr_exp;        /* bias-corrected step size lr_t = lr_q16 * 2^-(16 + lr_exp) */
  uint32_t beta1_q16, beta2_q16;  /* Q0.16 */
  uint32_t eps_q16, eps_exp;      /* eps = eps_q16 * 2^-(16 + eps_exp) */
} lpk_adam_hyper;

int lpk_adam_step(lpk_tensor_list* list,
                  const int32_t* fl_theta_in, const int32_t* fl_theta_out,
                  const int32_t* fl_mom_in, const int32_t* fl_mom_out,
                  const int32_t* fl_sec_in, const int32_t* fl_sec_out, const int32_t* fl_grad,
                  const lpk_adam_hyper* hyper /* host */,
                  uint64_t* vmax_out, uint64_t* mmax_out, uint64_t* umax_out, uint32_t* status, void* stream);

/*
 * The same ADAM step fed from the fp32 gradients (Sections 1, 2, 4): exactly
 * lpk_quantize_tensor(LPK_SEL_GRAD, fl_grad) followed by lpk_adam_step, in ONE pass that reads desc.src_f32,
 * quantizes each gradient in registers and never touches desc.grad.  Results are bit-identical to the two-call
 * sequence.  Every non-empty tensor needs src_f32, a momentum and a second-moment buffer (else INVALID_ARG).
 */
int lpk_adam_step_f32grad(lpk_tensor_list* list,
                          const int32_t* fl_theta_in, const int32_t* fl_theta_out,
                          const int32_t* fl_mom_in, const int32_t* fl_mom_out,
                          const int32_t* fl_sec_in, const int32_t* fl_sec_out, const int32_t* fl_grad,
                          const lpk_adam_hyper* hyper /* host */,
                          uint64_t* vmax_out, uint64_t* mmax_out, uint64_t* umax_out, uint32_t* status, void* stream);

/*
 * Bit-width guideline for the last fully-connected layer (Section 3, eq. 4-5): the smallest width BW with
 *   alpha / (n_classes - 1) >= 2^-(BW - 1),
 * i.e. the sum of the round-off parts of the softmax gradient stays below alpha.  Host-only, no device
 * access.  alpha_q16 = alpha * 65536 in (0, 65535] (the paper recommends alpha = 0.5 -> 32768).
 * Returns BW >= 2, or LPK_ERR_INVALID_ARG for n_classes < 2 or alpha_q16 outside (0, 65535].
 * Examples at alpha = 0.5: 10 classes -> 6, 58 -> 8, 1000 -> 12 bits.
 */
int lpk_classifier_min_bits(uint32_t n_classes, uint32_t alpha_q16);

/* Static text for a return code ("ok", "invalid argument", ...). Never NULL. */
const char* lpk_error_string(int code);

/* Library version, major * 10000 + minor * 100 + patch. */
int lpk_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LPK_H */

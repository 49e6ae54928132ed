/*
 * lpk_ref.c -- CPU oracle for the low-precision SGD update with Kahan summation
 * ("lazy update") over dynamic fixed-point (DFX) parameters.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, one-element-at-a-time
 * statement of what the update computes, used only to check the GPU library
 * and to time a CPU baseline.  It shares no code with the GPU path and the
 * GPU path never calls it.
 *
 * What it follows (paper: "Training Deep Neural Network in Limited Precision"):
 *   - Section 2, Algorithm 1 (lazy update): accumulate the step into an extra
 *     parameter, move theta by the part of it that theta's precision can hold,
 *     keep the remainder.
 *   - Section 2, Figure 1: parameter, gradient and accumulator share one
 *     decimal-point axis; with k overlapping bits the parameter is effectively
 *     m + n - 2 - k bits wide.
 *   - Section 1 (hardware model): 8/16-bit dynamic fixed point, uniform linear
 *     quantization, no stochastic rounding.
 *   - Section 6: a tensor's exponent is found by scanning its maximum.
 *
 * Notation.  DFX(W, fl) is a two's-complement integer q of W in {8,16} bits
 * whose real value is q * 2^-fl.  qmax = 2^(W-1)-1, qmin = -2^(W-1).
 * RNE = round to nearest, ties to even.  The compensation c stored here is the
 * NEGATIVE of Algorithm 1's acc, so theta + c is the "virtual" parameter.
 *
 * Readings where the paper is silent (rounding mode, saturation, position of
 * the accumulator's decimal point, the fractional-length rule, the learning
 * rate format, weight decay) are fixed as follows and nowhere else:
 *   rounding: RNE everywhere;  overflow: saturate at store, intermediates wide;
 *   c lives on grid fl_theta + d (d = W_c - 1 means no overlapping bit, k = 0);
 *   fraclen: the largest fl at which the tensor's own maximum does not saturate;
 *   lr and weight decay: unsigned Q0.16 integers.
 *
 * Every quantity is an exact integer; __int128 is used so that no intermediate
 * can overflow inside the documented domain (fraclens in [-64,64], 0<=d<=24,
 * |fl_out - fl_in| <= 15, lr_q16, wd_q16 <= 65535).
 *
 * Parity pins (tests/, CPU only): exact-rational brute force on tiny tensors,
 * the Kahan conservation invariant, the quarter-LSB worked example, the
 * effective-width closed form, torch.round cross-check for quantization,
 * definition-level brute force for the fraclen rule.
 */
#include <stdint.h>
#include <string.h>
#include <stddef.h>
#include <math.h>
#include <float.h>

typedef __int128 wide;

#define LPK_REF_OK            0
#define LPK_REF_ERR_ARG     (-1)

#define STATUS_NONFINITE     1u   /* a NaN or Inf was seen in fp32 input        */
#define STATUS_DOMAIN        2u   /* a fraclen / shift outside the domain; the
                                     tensor was left untouched                 */

#define FL_MIN (-64)
#define FL_MAX   64
#define D_MAX    24
#define DELTA_MAX 15

static const wide HUGE_W = (wide)1 << 100;   /* stands for "beyond every bound used here" */
static const wide CAP40  = (wide)1 << 40;

/* ---------- exact helpers ------------------------------------------------ */

/* RNE(x * 2^-k) for any integer k, as if in unbounded integers.
 * Callers keep |x| < 2^98.  For k <= -60 and x != 0 the exact value has
 * magnitude >= 2^60, which exceeds every clamp applied afterwards (2^40 cap,
 * 16-bit saturation), so +-2^100 is returned in its place. */
static wide rescale(wide x, int k)
{
    if (x == 0) return 0;
    if (k <= 0) {
        if (k <= -60) return x > 0 ? HUGE_W : -HUGE_W;
        return x * ((wide)1 << (-k));                /* exact */
    }
    if (k >= 100) return 0;                          /* |x| 2^-k < 1/4 */
    wide p = (wide)1 << k;
    wide q = x / p;                                  /* truncates toward zero */
    wide r = x % p;
    if (r < 0) { r += p; q -= 1; }                   /* now x = q p + r, 0 <= r < p (floor) */
    if (2 * r > p || (2 * r == p && (q & 1))) q += 1;
    return q;
}

static wide clampw(wide x, wide lo, wide hi) { return x < lo ? lo : (x > hi ? hi : x); }

static wide rescale_cap(wide x, int k) { return clampw(rescale(x, k), -CAP40, CAP40); }

static wide qmax_of(int bits) { return ((wide)1 << (bits - 1)) - 1; }
static wide qmin_of(int bits) { return -((wide)1 << (bits - 1)); }
static wide sat(wide x, int bits) { return clampw(x, qmin_of(bits), qmax_of(bits)); }

static int bits_ok(int bits) { return bits == 8 || bits == 16; }

static wide load_q(const void *p, uint64_t i, int bits)
{
    return bits == 8 ? (wide)((const int8_t *)p)[i] : (wide)((const int16_t *)p)[i];
}
static void store_q(void *p, uint64_t i, int bits, wide v)
{
    if (bits == 8) ((int8_t *)p)[i] = (int8_t)v; else ((int16_t *)p)[i] = (int16_t)v;
}

/* An fp32 is the exact dyadic rational (-1)^neg * m * 2^ex.  kind: 0 finite, 1 inf, 2 nan. */
static int decompose_f32(float x, int *neg, wide *m, int *ex)
{
    uint32_t b; memcpy(&b, &x, 4);
    uint32_t E = (b >> 23) & 0xFFu, frac = b & 0x7FFFFFu;
    *neg = (int)(b >> 31);
    if (E == 0xFFu) { *m = 0; *ex = 0; return frac ? 2 : 1; }
    if (E == 0) { *m = frac; *ex = -149; }               /* zero / subnormal */
    else        { *m = (wide)(frac | 0x800000u); *ex = (int)E - 150; }
    return 0;
}

/* ---------- fractional-length rule --------------------------------------- */

/* fl*(M, W): the LARGEST integer fl with RNE(M * 2^fl) <= qmax, for M = m * 2^ex > 0,
 * found by trying candidates from fine to coarse; the result is then clamped to
 * [FL_MIN, FL_MAX].  (Scanning the maximum to choose the exponent: Section 6;
 * the rule itself is this build's reading -- the widest-precision grid on which
 * the tensor's own maximum does not saturate.) */
static int fraclen_of_max(wide m, int ex, int bits)
{
    int fl;
    for (fl = 400; fl > -400; --fl)
        if (rescale(m, -(ex + fl)) <= qmax_of(bits)) break;
    if (fl > FL_MAX) fl = FL_MAX;
    if (fl < FL_MIN) fl = FL_MIN;
    return fl;
}

/* max|x| over an fp32 tensor -> fraclen for a W-bit grid.
 * Zero tensor (or n == 0) -> fl_default.  Any NaN/Inf -> FL_MIN and the
 * non-finite status bit. */
int lpk_ref_select_fraclen_f32(const float *x, uint64_t n, int bits, int32_t fl_default,
                               int32_t *fl_out, uint32_t *status)
{
    if (!bits_ok(bits) || !fl_out || (n && !x)) return LPK_REF_ERR_ARG;
    float best = 0.0f; int nonfinite = 0;
    for (uint64_t i = 0; i < n; ++i) {
        float a = fabsf(x[i]);                 /* exact */
        if (!(a <= FLT_MAX)) { nonfinite = 1; continue; }   /* NaN or Inf */
        if (a > best) best = a;                /* exact comparison */
    }
    int neg, best_ex; wide best_m;
    decompose_f32(best, &neg, &best_m, &best_ex);
    if (nonfinite) {
        *fl_out = FL_MIN;
        if (status) *status |= STATUS_NONFINITE;
        return LPK_REF_OK;
    }
    *fl_out = best_m == 0 ? fl_default : fraclen_of_max(best_m, best_ex, bits);
    return LPK_REF_OK;
}

/* Re-selection from the running maximum of the compensated sum (Section 6:
 * exponent from the history of maxima, here with a one-step lag):
 * M = vmax * 2^-vmax_fl.  vmax == 0 keeps fl_default.  The result is clamped
 * to fl_default +- DELTA_MAX (the next update can move the grid by at most
 * that much) and to [FL_MIN, FL_MAX]. */
int lpk_ref_select_fraclen_vmax(uint64_t vmax, int32_t vmax_fl, int bits, int32_t fl_default,
                                int32_t *fl_out, uint32_t *status)
{
    if (!bits_ok(bits) || !fl_out) return LPK_REF_ERR_ARG;
    if (vmax_fl < FL_MIN || vmax_fl > FL_MAX + D_MAX || fl_default < FL_MIN || fl_default > FL_MAX) {
        *fl_out = fl_default;
        if (status) *status |= STATUS_DOMAIN;
        return LPK_REF_OK;
    }
    if (vmax == 0) { *fl_out = fl_default; return LPK_REF_OK; }
    int fl = fraclen_of_max((wide)vmax, -vmax_fl, bits);
    if (fl > fl_default + DELTA_MAX) fl = fl_default + DELTA_MAX;
    if (fl < fl_default - DELTA_MAX) fl = fl_default - DELTA_MAX;
    if (fl > FL_MAX) fl = FL_MAX;
    if (fl < FL_MIN) fl = FL_MIN;
    *fl_out = fl;
    return LPK_REF_OK;
}

/* ---------- quantization -------------------------------------------------- */

/* q_i = sat_W(RNE(x_i * 2^fl)): uniform linear quantization, no stochastic
 * rounding (Section 1).  NaN -> 0, +-Inf -> qmax/qmin, both raise the
 * non-finite status bit.  fl outside [FL_MIN, FL_MAX]: nothing written,
 * domain status bit. */
int lpk_ref_quantize(const float *x, uint64_t n, int bits, int32_t fl, void *dst, uint32_t *status)
{
    if (!bits_ok(bits) || (n && (!x || !dst))) return LPK_REF_ERR_ARG;
    if (n == 0) return LPK_REF_OK;        /* an empty tensor is a no-op: there is no element whose grid could be wrong */
    if (fl < FL_MIN || fl > FL_MAX) { if (status) *status |= STATUS_DOMAIN; return LPK_REF_OK; }
    for (uint64_t i = 0; i < n; ++i) {
        int neg, ex; wide m;
        int kind = decompose_f32(x[i], &neg, &m, &ex);
        wide q;
        if (kind == 2)      { q = 0;                                   if (status) *status |= STATUS_NONFINITE; }
        else if (kind == 1) { q = neg ? qmin_of(bits) : qmax_of(bits); if (status) *status |= STATUS_NONFINITE; }
        else                 q = sat(rescale(neg ? -m : m, -(ex + fl)), bits);
        store_q(dst, i, bits, q);
    }
    return LPK_REF_OK;
}

/* ---------- the update ----------------------------------------------------- */

/*
 * One lazy-update step over one tensor, in place.
 *
 *   theta : DFX(theta_bits, fl_in) on entry, DFX(theta_bits, fl_out) on exit
 *   comp  : c = -acc, DFX(comp_bits, fl_in + d) on entry, (fl_out + d) on exit;
 *           NULL = plain SGD without the accumulator (eq. 1)
 *   grad  : DFX(grad_bits, fl_g)
 *   lr_q, wd_q : Q0.16 (wd_q == 0: no decay)
 *   vmax  : max_i |v_i| of the compensated sum on grid fl_in + d (may be NULL)
 *
 * Per element, with F = fl_in + d the working grid (units: LSBs of c):
 *   s_g = cap( RNE( -lr_q * g * 2^-(fl_g + 16 - F) ) )      step on c's grid   [Alg. 1, 1st assignment]
 *   s_w = cap( RNE( -lr_q * wd_q * theta * 2^-(32 - d) ) )  decay, rounded separately
 *   v   = theta * 2^d + c + s_g + s_w                       kept wide (never cut to comp_bits)
 *   theta' = sat( RNE( v on the fl_out grid ) )             [Alg. 1, 2nd assignment]
 *   c'     = sat( RNE( (v - theta') on the fl_out + d grid ) )   [Alg. 1, 3rd assignment]
 *   store theta', c'                                        [Alg. 1, 4th assignment]
 */
int lpk_ref_kahan_sgd_step(void *theta, void *comp, const void *grad, uint64_t n,
                           int theta_bits, int comp_bits, int grad_bits, int d,
                           int32_t fl_in, int32_t fl_out, int32_t fl_g,
                           uint32_t lr_q, uint32_t wd_q,
                           uint64_t *vmax, uint32_t *status)
{
    if (!bits_ok(theta_bits) || !bits_ok(grad_bits) || (comp && !bits_ok(comp_bits))) return LPK_REF_ERR_ARG;
    if (n && (!theta || !grad)) return LPK_REF_ERR_ARG;
    if (lr_q > 65535u || wd_q > 65535u) return LPK_REF_ERR_ARG;
    if (!comp) d = 0;
    if (vmax) *vmax = 0;
    if (n == 0) return LPK_REF_OK;                    /* an empty tensor is a no-op: nothing to flag */
    int delta = fl_out - fl_in;
    if (fl_in < FL_MIN || fl_in > FL_MAX || fl_out < FL_MIN || fl_out > FL_MAX ||
        fl_g < FL_MIN || fl_g > FL_MAX || d < 0 || d > D_MAX ||
        delta > DELTA_MAX || delta < -DELTA_MAX) {
        if (status) *status |= STATUS_DOMAIN;
        return LPK_REF_OK;
    }
    const int F = fl_in + d;
    const int u = delta > 0 ? delta : 0;
    const int k_theta = d + u - delta;          /* >= d >= 0 */
    wide vm = 0;
    for (uint64_t i = 0; i < n; ++i) {
        wide th = load_q(theta, i, theta_bits);
        wide c  = comp ? load_q(comp, i, comp_bits) : 0;
        wide g  = load_q(grad, i, grad_bits);

        wide s = rescale_cap(-(wide)lr_q * g, fl_g + 16 - F);
        if (wd_q) s += rescale_cap(-(wide)lr_q * (wide)wd_q * th, fl_in + 32 - F);

        wide v = th * ((wide)1 << d) + c + s;
        wide av = v < 0 ? -v : v;
        if (av > vm) vm = av;

        wide vG  = v * ((wide)1 << u);
        wide thn = sat(rescale(vG, k_theta), theta_bits);
        store_q(theta, i, theta_bits, thn);
        if (comp) {
            wide r = vG - thn * ((wide)1 << k_theta);
            store_q(comp, i, comp_bits, sat(rescale(r, k_theta - d), comp_bits));
        }
    }
    if (vmax) *vmax = (uint64_t)vm;
    return LPK_REF_OK;
}

/* ---------- momentum SGD with the lazy update inside ------------------------------------------------------- */

/*
 * Section 4 trains most networks with the momentum optimizer (mu = 0.9) "with the lazy update implemented in
 * the optimizer", with an INT8 or INT16 velocity; the paper does not write the combination out.  Reading taken
 * here (the textbook heavy-ball form with the learning rate inside the velocity):
 *
 *     m <- mu * m - lr * (g + wd * theta)          velocity, a third DFX tensor with its own fraclen
 *     theta <- theta + m                           through Algorithm 1: acc takes the step m
 *
 * In fixed point, with G = fl_m_out + 16 the working grid of the velocity (16 guard bits below its LSB):
 *     w  = RNE(mu_q * m on grid G)                           (exact unless the velocity grid gets coarser)
 *        + cap(RNE(-lr_q * g on grid G)) + cap(RNE(-lr_q * wd_q * theta on grid G))
 *     m' = sat(RNE(w / 2^16))                                 stored on grid fl_m_out
 *     s  = cap(RNE(m' on grid F))                             F = fl_in + d, then exactly the lazy update with this s
 *     mmax = max |RNE(w / 2^16)|  (the velocity before saturation, on grid fl_m_out), vmax = max |v| (on grid F)
 */
int lpk_ref_momentum_sgd_step(void *theta, void *comp, void *mom, const void *grad, uint64_t n,
                              int theta_bits, int comp_bits, int mom_bits, int grad_bits, int d,
                              int32_t fl_in, int32_t fl_out, int32_t fl_m_in, int32_t fl_m_out, int32_t fl_g,
                              uint32_t lr_q, uint32_t mu_q, uint32_t wd_q,
                              uint64_t *vmax, uint64_t *mmax, uint32_t *status)
{
    if (!bits_ok(theta_bits) || !bits_ok(grad_bits) || !bits_ok(mom_bits) || (comp && !bits_ok(comp_bits))) return LPK_REF_ERR_ARG;
    if (n && (!theta || !grad || !mom)) return LPK_REF_ERR_ARG;
    if (lr_q > 65535u || wd_q > 65535u || mu_q > 65535u) return LPK_REF_ERR_ARG;
    if (!comp) d = 0;
    if (vmax) *vmax = 0;
    if (mmax) *mmax = 0;
    if (n == 0) return LPK_REF_OK;                    /* an empty tensor is a no-op: nothing to flag */
    int delta = fl_out - fl_in, delta_m = fl_m_out - fl_m_in;
    if (fl_in < FL_MIN || fl_in > FL_MAX || fl_out < FL_MIN || fl_out > FL_MAX || fl_g < FL_MIN || fl_g > FL_MAX ||
        fl_m_in < FL_MIN || fl_m_in > FL_MAX || fl_m_out < FL_MIN || fl_m_out > FL_MAX ||
        d < 0 || d > D_MAX || delta > DELTA_MAX || delta < -DELTA_MAX || delta_m > DELTA_MAX || delta_m < -DELTA_MAX) {
        if (status) *status |= STATUS_DOMAIN;
        return LPK_REF_OK;
    }
    const int F = fl_in + d, G = fl_m_out + 16;
    const int u = delta > 0 ? delta : 0;
    const int k_theta = d + u - delta;
    wide vm = 0, wm = 0;
    for (uint64_t i = 0; i < n; ++i) {
        wide th = load_q(theta, i, theta_bits);
        wide c  = comp ? load_q(comp, i, comp_bits) : 0;
        wide m  = load_q(mom, i, mom_bits);
        wide g  = load_q(grad, i, grad_bits);

        /* velocity: mu_q*m sits on grid fl_m_in + 16, lr_q*g on fl_g + 16, lr_q*wd_q*theta on fl_in + 32 */
        wide w = rescale((wide)mu_q * m, (fl_m_in + 16) - G);
        w += rescale_cap(-(wide)lr_q * g, (fl_g + 16) - G);
        if (wd_q) w += rescale_cap(-(wide)lr_q * (wide)wd_q * th, (fl_in + 32) - G);
        wide mq = rescale(w, 16);                 /* the new velocity before saturation */
        wide aw = mq < 0 ? -mq : mq;
        if (aw > wm) wm = aw;
        wide mn = sat(mq, mom_bits);
        store_q(mom, i, mom_bits, mn);

        /* the new velocity is the step handed to the accumulator (Algorithm 1, 1st assignment) */
        wide s = rescale_cap(mn, fl_m_out - F);
        wide v = th * ((wide)1 << d) + c + s;
        wide av = v < 0 ? -v : v;
        if (av > vm) vm = av;
        wide vG  = v * ((wide)1 << u);
        wide thn = sat(rescale(vG, k_theta), theta_bits);
        store_q(theta, i, theta_bits, thn);
        if (comp) {
            wide r = vG - thn * ((wide)1 << k_theta);
            store_q(comp, i, comp_bits, sat(rescale(r, k_theta - d), comp_bits));
        }
    }
    if (vmax) *vmax = (uint64_t)vm;
    if (mmax) *mmax = (uint64_t)wm;
    return LPK_REF_OK;
}

/* ---------- ADAM with the lazy update inside ------------------------------------------------------------------ */

/* floor(sqrt(a)) for 0 <= a < 2^62, one result bit at a time: keep the bit when the square still fits. */
static wide isqrt_floor(wide a)
{
    wide r = 0;
    for (int b = 31; b >= 0; --b) {
        wide t = r + ((wide)1 << b);
        if (t * t <= a) r = t;
    }
    return r;
}

/* RNE(num / den) for integers, den > 0: floor quotient, then compare twice the remainder with den. */
static wide div_rne(wide num, wide den)
{
    wide q = num / den, r = num % den;
    if (r < 0) { r += den; q -= 1; }                 /* num = q den + r, 0 <= r < den */
    if (2 * r > den || (2 * r == den && (q & 1))) q += 1;
    return q;
}

/*
 * Section 4 trains the SVHN network, the GANs and the LSTM with the ADAM optimizer in INT16 "with the lazy update
 * implemented in the optimizer"; the paper names only the hyper-parameters (beta1, beta2, epsilon, learning rate)
 * and that 16 bits are needed because of beta2.  Reading taken here: the textbook rule
 *
 *     m <- beta1 m + (1 - beta1) g        u <- beta2 u + (1 - beta2) g^2        theta <- theta - lr_t m / (sqrt(u) + eps)
 *
 * with the bias corrections folded into the step size lr_t = lr sqrt(1 - beta2^t) / (1 - beta1^t) by the caller,
 * m and u two DFX state tensors with fraclens of their own, and the step handed to Algorithm 1's accumulator.
 * Constants: beta1, beta2 as Q0.16 (their complements are 65536 - beta); lr_t = lr_q * 2^-(16 + lr_exp) and
 * eps = eps_q * 2^-(16 + eps_exp) with 16-bit lr_q, eps_q and 0 <= lr_exp, eps_exp <= 48.
 *
 * In fixed point (every RNE as if in unbounded integers, cap = clamp to +-2^40):
 *     wM = RNE(b1 m on grid Gm) + cap(RNE((65536 - b1) g on Gm)),   Gm = fl_m_out + 16
 *     mq = RNE(wM / 2^16);  m' = sat(mq);  mmax = max |mq|
 *     wU = RNE(b2 u on grid Gu) + cap(RNE((65536 - b2) g^2 on Gu)), Gu = fl_u_out + 16
 *     uq = RNE(wU / 2^16);  u' = clamp(uq, 0, qmax);  umax = max(uq, 0) over the tensor
 *     rt = floor(sqrt(u' 2^(24 + p))),  p = parity of fl_u_out: the root on grid R = (fl_u_out + 24 + p) / 2
 *     den = max(rt + min(RNE(eps on grid R), 2^30), 1)
 *     s  = cap(RNE(-lr_q m' 2^e / den)),  e = F + R - 16 - lr_exp - fl_m_out,  F = fl_in + d
 *   then exactly the lazy update with this s.  e > 20 is outside the domain (the tensor is skipped).
 */
int lpk_ref_adam_step(void *theta, void *comp, void *mom, void *sec, const void *grad, uint64_t n,
                      int theta_bits, int comp_bits, int mom_bits, int sec_bits, int grad_bits, int d,
                      int32_t fl_in, int32_t fl_out, int32_t fl_m_in, int32_t fl_m_out,
                      int32_t fl_u_in, int32_t fl_u_out, int32_t fl_g,
                      uint32_t lr_q, uint32_t lr_exp, uint32_t b1_q, uint32_t b2_q, uint32_t eps_q, uint32_t eps_exp,
                      uint64_t *vmax, uint64_t *mmax, uint64_t *umax, uint32_t *status)
{
    if (!bits_ok(theta_bits) || !bits_ok(grad_bits) || !bits_ok(mom_bits) || !bits_ok(sec_bits) ||
        (comp && !bits_ok(comp_bits))) return LPK_REF_ERR_ARG;
    if (n && (!theta || !grad || !mom || !sec)) return LPK_REF_ERR_ARG;
    if (lr_q > 65535u || b1_q > 65535u || b2_q > 65535u || eps_q > 65535u || lr_exp > 48u || eps_exp > 48u) return LPK_REF_ERR_ARG;
    if (!comp) d = 0;
    if (vmax) *vmax = 0;
    if (mmax) *mmax = 0;
    if (umax) *umax = 0;
    if (n == 0) return LPK_REF_OK;                    /* an empty tensor is a no-op: nothing to flag */
    const int delta = fl_out - fl_in, delta_m = fl_m_out - fl_m_in, delta_u = fl_u_out - fl_u_in;
    const int F = fl_in + d, Gm = fl_m_out + 16, Gu = fl_u_out + 16;
    const int par = ((fl_u_out % 2) + 2) % 2;
    const int R = (fl_u_out + 24 + par) / 2;                      /* exact: the numerator is even */
    const int e = F + R - 16 - (int)lr_exp - fl_m_out;
    if (fl_in < FL_MIN || fl_in > FL_MAX || fl_out < FL_MIN || fl_out > FL_MAX || fl_g < FL_MIN || fl_g > FL_MAX ||
        fl_m_in < FL_MIN || fl_m_in > FL_MAX || fl_m_out < FL_MIN || fl_m_out > FL_MAX ||
        fl_u_in < FL_MIN || fl_u_in > FL_MAX || fl_u_out < FL_MIN || fl_u_out > FL_MAX ||
        d < 0 || d > D_MAX || delta > DELTA_MAX || delta < -DELTA_MAX || delta_m > DELTA_MAX || delta_m < -DELTA_MAX ||
        delta_u > DELTA_MAX || delta_u < -DELTA_MAX || e > 20) {
        if (status) *status |= STATUS_DOMAIN;
        return LPK_REF_OK;
    }
    const int u_shift = delta > 0 ? delta : 0;
    const int k_theta = d + u_shift - delta;
    wide eps_R = rescale((wide)eps_q, 16 + (int)eps_exp - R);
    if (eps_R > ((wide)1 << 30)) eps_R = (wide)1 << 30;
    wide vm = 0, wm = 0, um = 0;
    for (uint64_t i = 0; i < n; ++i) {
        wide th = load_q(theta, i, theta_bits);
        wide c  = comp ? load_q(comp, i, comp_bits) : 0;
        wide m  = load_q(mom, i, mom_bits);
        wide u  = load_q(sec, i, sec_bits);
        wide g  = load_q(grad, i, grad_bits);

        /* first moment: b1*m sits on grid fl_m_in + 16, (1 - b1)*g on fl_g + 16 */
        wide wM = rescale((wide)b1_q * m, (fl_m_in + 16) - Gm);
        wM += rescale_cap((wide)(65536u - b1_q) * g, (fl_g + 16) - Gm);
        wide mq = rescale(wM, 16);
        wide am = mq < 0 ? -mq : mq;
        if (am > wm) wm = am;
        wide mn = sat(mq, mom_bits);
        store_q(mom, i, mom_bits, mn);

        /* second moment: b2*u sits on grid fl_u_in + 16, (1 - b2)*g^2 on 2 fl_g + 16 */
        wide wU = rescale((wide)b2_q * u, (fl_u_in + 16) - Gu);
        wU += rescale_cap((wide)(65536u - b2_q) * g * g, (2 * fl_g + 16) - Gu);
        wide uq = rescale(wU, 16);
        if (uq > um) um = uq;
        wide un = clampw(uq, 0, qmax_of(sec_bits));
        store_q(sec, i, sec_bits, un);

        /* the step: -lr_t * m' / (sqrt(u') + eps) on grid F */
        wide rt  = isqrt_floor(un * ((wide)1 << (24 + par)));
        wide den = rt + eps_R;
        if (den < 1) den = 1;
        wide num = -(wide)lr_q * mn;
        wide s;
        if (e >= 0) s = div_rne(num * ((wide)1 << e), den);
        else if (e > -80) s = div_rne(num, den * ((wide)1 << (-e)));
        else s = 0;                                   /* |num| < 2^31 against a divisor >= 2^80 */
        s = clampw(s, -CAP40, CAP40);

        wide v = th * ((wide)1 << d) + c + s;
        wide av = v < 0 ? -v : v;
        if (av > vm) vm = av;
        wide vG  = v * ((wide)1 << u_shift);
        wide thn = sat(rescale(vG, k_theta), theta_bits);
        store_q(theta, i, theta_bits, thn);
        if (comp) {
            wide r = vG - thn * ((wide)1 << k_theta);
            store_q(comp, i, comp_bits, sat(rescale(r, k_theta - d), comp_bits));
        }
    }
    if (vmax) *vmax = (uint64_t)vm;
    if (mmax) *mmax = (uint64_t)wm;
    if (umax) *umax = (uint64_t)um;
    return LPK_REF_OK;
}

/* ---------- classifier bit-width guideline (Section 3, eq. 4) ------------------------------------------------ */

/* Smallest BW for which  alpha / (|class| - 1) >= 2^-(BW-1)  holds, alpha = alpha_q16 / 65536, found by
 * testing the inequality itself for BW = 2, 3, ... in exact integers:
 *   alpha_q16 * 2^(BW-1) >= (|class| - 1) * 65536.                                                         */
int lpk_ref_classifier_min_bits(uint32_t n_classes, uint32_t alpha_q16)
{
    if (n_classes < 2 || alpha_q16 == 0 || alpha_q16 > 65535u) return LPK_REF_ERR_ARG;
    for (int bw = 2; bw < 120; ++bw) {
        wide lhs = (wide)alpha_q16 * ((wide)1 << (bw - 1));
        wide rhs = (wide)(n_classes - 1) * 65536;
        if (lhs >= rhs) return bw;
    }
    return LPK_REF_ERR_ARG;
}

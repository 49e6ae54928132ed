// ADAM with the lazy update inside (paper, Section 4: the ADAM optimizer in INT16 with Algorithm 1 implemented in
// the optimizer).  One fused launch over every tile of every tensor:
//
//   wM = RNE(b1*m on grid Gm) + cap(RNE((1-b1)*g on Gm));   mq = RNE(wM / 2^16);  m' = sat(mq)
//   wU = RNE(b2*u on grid Gu) + cap(RNE((1-b2)*g^2 on Gu)); uq = RNE(wU / 2^16);  u' = clamp(uq, 0, qmax)
//   rt = floor(sqrt(u' * 2^(24+p)));  den = max(rt + eps_R, 1);  s = cap(RNE(-lr*m'*2^e / den))
//   then Algorithm 1 with step s.
//
// Arithmetic, general route: everything runs on the fp64 unit, and every value is exact.  Each intermediate above is an integer
// below 2^53 times a power of two (16-bit words times 17-bit constants, 2^40 caps, shifts of the documented
// domain), so products, sums and scalings by powers of two are exact in binary64 and v_rndne_f64 is the
// round-to-nearest-even of the definition, for every shift direction, without a branch.  The two inexact
// operations are repaired with exact residuals: the root by the sign of fma(r, r, -A), the quotient by the
// remainder fma(-q, den, num) compared with half the divisor (ties to even).
//
// The usual case takes a shorter route with the same results ("fast": both moment grids standing still, the first
// moment's grid at most eight bits finer than the gradient's, a step below 2^22 accumulator LSBs).  There the
// first moment b1*m + (1-b1)*g*2^sh = 65536*m - (1-b1)*(m - g*2^sh) is ONE fp32 fused multiply-add onto the
// constant 1.5*2^39 + 65536*m (ulp 2^16): its single IEEE rounding is the RNE at bit 16 and the new moment is read
// from the significand.  The second moment is a 24-bit multiply-add and an integer round-half-even around one
// fp64 FMA (the rounding of (1-b2)*g^2 onto u's guard-bit grid).  The root is the fp32 square root nudged below the
// true root, truncated, and repaired upwards by the sign of one fp32 FMA (R*R - A is formed exactly inside it).
// Only the quotient stays on the fp64 unit, without the Newton step: a quotient below 2^22 from the reciprocal's
// documented 2^-23 relative accuracy is less than one away from the exact one, which is what the remainder test
// repairs.  12 fp64 instructions per parameter instead of 46.
//
// Same work distribution as the plain update (persistent wavefronts over the tile table, non-temporal vector
// accesses) for int16 moments and gradients on 16-byte aligned buffers -- in 1024-element rows with a cross-lane
// swap for int8 theta and accumulator with int16 gradients (see ARow), in groups of 8 consecutive elements per lane
// otherwise; anything else goes element by element through the same arithmetic.  Gradients come from the int16 array or, in a second kernel instance, from the
// fp32 source, quantized in registers.
#include "step_common.hpp"

#ifndef LPK_ADAM_E
#define LPK_ADAM_E 8                   // consecutive elements per lane per group (4 or 8)
#endif
#ifndef LPK_ADAM_GROUPS
#define LPK_ADAM_GROUPS 4              // groups in flight per lane (measured: 2, 6, 8, 16 are slower for one or both gradient sources)
#endif
#ifndef LPK_ADAM_ROWS
#define LPK_ADAM_ROWS 2                // int8 theta and accumulator, int16 gradients: 1024-element rows in flight per wave (0: groups only;
                                       // 2 and 4 measure the same, 3 is slower; 4 needs more than 256 registers)
#endif
#ifndef LPK_ADAM_WAVES_PER_SIMD
#define LPK_ADAM_WAVES_PER_SIMD 1      // lower bound handed to the register allocator (no cap at 256 VGPRs: nothing spills; the kernel
                                       // still fits two waves per SIMD, which is how it is launched)
#endif

namespace lpk {

struct AdamParams {
  int    path;                     // 0 skip (-1: skip, but look at the fp32 gradients), 1 element by element, 2 vector
  int    wt, wc, wg, wm, wu, has_comp;
  int    caps;                     // some 2^40 cap may bind
  int    exact3;                   // a1, a2, a3 are integers (and no cap binds): three of the four products need no rounding
  double a1, a2, a3, a4;           // b1 * 2^-k1, (65536 - b1) * 2^-k2, b2 * 2^-k4, (65536 - b2) * 2^-k5
  double qmin_m, qmax_m, qmax_u;
  double ascale;                   // 2^(24 + p): radicand scale
  double eps_r;                    // eps on the root's grid, at most 2^30
  double nlr;                      // -lr * 2^e
  Alg1Wide wa;                     // last stage of Algorithm 1 in fp64
  float  gscale, glo, ghi;         // fp32 gradient source: 2^fl_g and the rails of the gradient width
  // 32-bit tail (int8 theta, fixed grid, every |intermediate| of Algorithm 1 below 2^22): as in the plain update,
  // fma(v, 2^-d, 1.5 * 2^23) rounds v onto theta's grid and one 24-bit multiply-add forms the residual
  int    tail;                     // kTailWide, kTailSmall (int8 accumulator, d <= 8) or kTailSmallBigD (int16 accumulator)
  int    d;
  Alg1Small sm;
  // fast route (see update_adam_fast)
  int    fast;
  int    neg2sh;                   // -2^sh, sh = fl_m_out - fl_g
  float  nc1_f;                    // -(65536 - b1)
  int    nc2;                      // -(65536 - b2)
  int    qmin_mi, qmax_mi, qmax_ui, eps_i;
  float  ascale_f;                 // 2^(24 + p)
};

enum { kTailWide = 0, kTailSmall = 1, kTailSmallBigD = 2 };

struct AdamTrack { double vm, mm, um; VTrack v, m; int umx; };     // fp64 route's maxima; 32-bit routes' extremes of v and mq, max of uq

__device__ __forceinline__ double cap_d() { return 1099511627776.0; }          // 2^40

// CAPS: whether a 2^40 cap can bind for this tensor's shifts (wave-uniform; almost never).
// EXACT3: b1 * 2^-k1, (1 - b1) * 2^-k2 and b2 * 2^-k4 are integers, as they are whenever the moments' grids stand
// still and the first moment's grid is not coarser than the gradient's: those three products are then integers
// already, their roundings are identities and are left out (never together with CAPS).
template <bool CAPS, int TAIL, bool EXACT3>
__device__ __forceinline__ void update_adam(const AdamParams& p, int th, int c, int m, int u, int g,
                                            int& tn, int& cn, int& mn, int& un, AdamTrack& tr)
{
  const double cap = 1099511627776.0;                       // 2^40
  const double gd = (double)g;
  // first moment
  double wm;
  if (EXACT3) {
    wm = __builtin_fma((double)m, p.a1, gd * p.a2);         // integers below 2^47: exact
  } else {
    const double t1 = __builtin_rint((double)m * p.a1);
    double t2 = __builtin_rint(gd * p.a2);
    if (CAPS) t2 = clampd(t2, -cap, cap);
    wm = t1 + t2;
  }
  const double mq = __builtin_rint(wm * 0x1p-16);
  tr.mm = __builtin_fmax(tr.mm, __builtin_fabs(mq));
  const double mnew = clampd(mq, p.qmin_m, p.qmax_m);
  // second moment
  double t4 = __builtin_rint(gd * gd * p.a4);
  if (CAPS) t4 = clampd(t4, -cap, cap);
  const double wu = EXACT3 ? __builtin_fma((double)u, p.a3, t4) : __builtin_rint((double)u * p.a3) + t4;
  const double uq = __builtin_rint(wu * 0x1p-16);
  tr.um = __builtin_fmax(tr.um, uq);
  const double unew = clampd(uq, 0.0, p.qmax_u);
  // Root of the new second moment on its fixed grid.  A is an integer below 2^40; the fp32 root of its fp32
  // rounding is within 0.2 of the true root (two relative errors of at most 2^-23 on a value below 2^20), so its
  // floor is off by at most one, which the signs of the exact residuals r^2 - A and (r + 1)^2 - A repair.
  const double A = unew * p.ascale;
  double r = __builtin_floor((double)__builtin_amdgcn_sqrtf((float)A));
  const double r1 = r + 1.0;
  // both residuals unconditionally (r^2 > A excludes (r + 1)^2 <= A), so the repair is two selects and no branch:
  // a branch here would keep the compiler from interleaving the sixteen elements' dependency chains
  const double r_dn = __builtin_fma(r, r, -A) > 0.0 ? 1.0 : 0.0, r_up = __builtin_fma(r1, r1, -A) <= 0.0 ? 1.0 : 0.0;
  r = (r - r_dn) + r_up;
  const double den = __builtin_fmax(r + p.eps_r, 1.0);
  // Step: RNE(num / den) with num = -lr m' 2^e (the power of two folded into the numerator: exact).  The
  // reciprocal seed (relative error below 2^-22) plus one Newton step leaves a relative error below 2^-43, so the
  // rounded product is within one of the exact rounded quotient whenever that is below 2^41 (larger ones end at
  // the cap regardless).  The exact remainder num - q den then decides: beyond half the divisor, or at half with
  // q odd, q moves by one towards the remainder's sign.  q's parity is read from the low word of q + 1.5 * 2^52.
  const double num = mnew * p.nlr;
  double x = __builtin_amdgcn_rcp(den);
  x = __builtin_fma(__builtin_fma(-den, x, 1.0), x, x);
  double q = __builtin_rint(num * x);
  const double rem = __builtin_fma(-q, den, num);
  const double t = __builtin_fabs(rem) * 2.0;
  const bool odd = (__double2loint(q + 6755399441055744.0) & 1) != 0;
  const bool adj = (t > den) | ((t == den) & odd);
  q += __hiloint2double(adj ? (0x3ff00000 | (__double2hiint(rem) & (int)0x80000000)) : 0, 0);
  const double s = CAPS ? clampd(q, -cap, cap) : q;
  mn = (int)mnew; un = (int)unew;
  // Algorithm 1 with this step
  if (TAIL != kTailWide) {
    const int v = (int)((unsigned)th << p.d) + c + (int)s;
    track_v(tr.v, v);
    alg1_small<(TAIL == kTailSmallBigD)>(p.sm, v, tn, cn);
    return;
  }
  alg1_wide(p.wa, th, c, s, tn, cn, tr.vm);
}

// The fast route (conditions in setup_adam; results identical to update_adam).
//   first moment:  wM = b1*m + c1*g*2^sh = 65536*m - c1*y with c1 = 65536 - b1, y = m - g*2^sh (|y| < 2^24, exact in
//     fp32).  fma(-c1, y, K + 65536*m) with K = 1.5*2^39 forms wM + K exactly and rounds it once to K's ulp, 2^16,
//     ties to even (K / 2^16 is even): the result is K + 2^16 * RNE(wM / 2^16).  K + 65536*m is K's bit pattern
//     plus m; the new moment is the result's bit pattern minus K's.  Needs |wM| < 2^38.
//   second moment: wU = b2*u + t4 = 65536*u + w with w = t4 - c2*u, t4 = RNE(g*g * a4) <= 2^30 from one fp64 FMA
//     onto 1.5*2^52 (whose low word is 0, so the sum's low word is t4).  RNE(wU / 2^16) is u plus w shifted right 16
//     with round-half-even, the parity taken from u + (w >> 16).  w is a signed word for u >= 0, an unsigned one for
//     u < 0 (see there); the result is clamped to [0, qmax] as the definition says, whatever sign u came with.
//   root:  A = u' * 2^(24+p) < 2^40 is exact in fp32.  v_sqrt_f32 is within 1 ulp; times (1 - 2^-21) it lies
//     strictly below the true root and less than 0.7 below it, so its truncation r0 is floor(root) or one less, and
//     floor(root) = r0 + [(r0+1)^2 <= A].  That sign is exact: the FMA forms (r0+1)^2 - A (an integer) before rounding.
//   quotient: q0 = RNE(num * rcp(den)) via the 1.5*2^52 constant (low word = q0).  |Q| < 0.99 * 2^22 and a reciprocal
//     within 2^-23 (relative) put num * rcp(den) less than 0.5 from Q, so q0 is less than 1 from Q; the exact remainder
//     num - q0*den against half the divisor (ties to even) moves q0 by at most one onto RNE(Q).
template <int TAIL>
__device__ __forceinline__ void update_adam_fast(const AdamParams& p, int th, int c, int m, int u, int g,
                                                 int& tn, int& cn, int& mn, int& un, AdamTrack& tr)
{
  constexpr int kMagic39 = ((127 + 39) << 23) | 0x400000;          // bits(1.5 * 2^39)
  const double kMagic52 = 6755399441055744.0;                      // 1.5 * 2^52
  // first moment
  const int y = mad_i24(g, p.neg2sh, m);
  const int mq = __float_as_int(__builtin_fmaf(p.nc1_f, (float)y, __int_as_float(kMagic39 + m))) - kMagic39;
  track_v(tr.m, mq);
  mn = med3_i32(mq, p.qmin_mi, p.qmax_mi);
  // second moment
  const int t4 = __double2loint(__builtin_fma((double)mad_i24(g, g, 0), p.a4, kMagic52));
  // w = t4 - c2*u lies in (-2^31, 2^30] for u >= 0 and in [0, 2^31 + 2^30) for u < 0 (a negative second moment is
  // not a state the optimizer reaches, but the definition covers every int16 input): a signed word in the first
  // case, an unsigned one in the second, and the 32-bit multiply-add is exact modulo 2^32 in both
  const int w = mad_i24(u, p.nc2, t4);
  const bool uneg = u < 0;
  const int lsb = (u + (uneg ? (int)((unsigned)w >> 16) : (w >> 16))) & 1;
  const unsigned ww = (unsigned)w + 0x7fffu + (unsigned)lsb;
  const int uq = u + (uneg ? (int)(ww >> 16) : ((int)ww >> 16));
  tr.umx = uq > tr.umx ? uq : tr.umx;
  un = med3_i32(uq, 0, p.qmax_ui);
  // root of the new second moment on its fixed grid
  const float Af = (float)un * p.ascale_f;
  const float r0 = __builtin_truncf(__builtin_amdgcn_sqrtf(Af) * 0.999999523162841796875f);     // 1 - 2^-21
  const float r1 = r0 + 1.0f;
  int den = (int)r0 + p.eps_i + (__builtin_fmaf(r1, r1, -Af) <= 0.0f ? 1 : 0);
  den = den > 1 ? den : 1;
  // step
  const double dend = (double)den;
  const double num = (double)mn * p.nlr;
  const double qm = __builtin_fma(num, __builtin_amdgcn_rcp(dend), kMagic52);
  const int q0 = __double2loint(qm);
  const double rem = __builtin_fma(-(qm - kMagic52), dend, num);
  const double t = __builtin_fabs(rem) + __builtin_fabs(rem);
  const bool adj = (t > dend) | ((t == dend) & ((q0 & 1) != 0));
  const int s = q0 + (adj ? ((__double2hiint(rem) >> 31) | 1) : 0);
  // Algorithm 1 with this step, in 32 bits
  const int v = (int)((unsigned)th << p.d) + c + s;
  track_v(tr.v, v);
  alg1_small<(TAIL == kTailSmallBigD)>(p.sm, v, tn, cn);
}

// Element-at-a-time tile: any alignment, any widths.  Lane l takes elements l, l+64, ...
template <bool CAPS, int GS>
__device__ __forceinline__ void tile_generic_adam(const AdamParams& p, const TensorDev& T, uint64_t off, uint32_t cnt, int lane, AdamTrack& tr,
                                                  uint32_t& ab)
{
  for (uint32_t j = lane; j < cnt; j += kWave) {
    const uint64_t i = off + j;
    const int th = load_elem(T.theta, i, p.wt);
    const int c  = p.has_comp ? load_elem(T.comp, i, p.wc) : 0;
    const int m  = load_elem(T.mom, i, p.wm);
    const int u  = load_elem(T.sec, i, p.wu);
    const int g  = GS == kGradF32 ? (int)quant_f32(((const float*)T.src)[i], p.gscale, p.glo, p.ghi, ab) : load_elem(T.grad, i, p.wg);
    int tn, cn, mn, un;
    update_adam<CAPS, kTailWide, false>(p, th, c, m, u, g, tn, cn, mn, un, tr);
    store_elem(T.theta, i, p.wt, tn);
    if (p.has_comp) store_elem(T.comp, i, p.wc, cn);
    store_elem(T.mom, i, p.wm, mn);
    store_elem(T.sec, i, p.wu, un);
  }
}

// E consecutive elements per lane; int16 moments and gradients.  With E = 8 every access of a wave is one contiguous
// run (dwordx4 for the 16-bit arrays, dwordx2 for 8-bit ones); four groups in flight at two waves per SIMD.
template <int E, int WT, int WC, int GS> struct AGroup {
  static constexpr int kG = GS == kGradF32 ? E / 4 : 1;          // gradient accesses: dwordx4 of fp32, or one of E int16
  static constexpr int kGN = GS == kGradF32 ? 4 : E / 2;
  DW<E * WT / 32> th;
  DW<E * WC / 32> c;
  DW<E / 2> m, u;
  DW<kGN> g[kG];
};

template <int E, int WT, int WC, int GS>
__device__ __forceinline__ void load_group_adam(AGroup<E, WT, WC, GS>& G, const TensorDev& T, uint64_t e)
{
  G.th = ld_dw<E * WT / 32>((const int8_t*)T.theta + e * (WT / 8));
  G.c  = ld_dw<E * WC / 32>((const int8_t*)T.comp + e * (WC / 8));
  G.m  = ld_dw<E / 2>((const int16_t*)T.mom + e);
  G.u  = ld_dw<E / 2>((const int16_t*)T.sec + e);
  if constexpr (GS == kGradF32) {
#pragma unroll
    for (int j = 0; j < E / 4; ++j) G.g[j] = ld_dw<4>((const float*)T.src + e + 4 * j);
  } else {
    G.g[0] = ld_dw<E / 2>((const int16_t*)T.grad + e);
  }
}

template <int E, int WT, int WC, bool CAPS, int TAIL, bool EXACT3, int GS, bool FAST>
__device__ __forceinline__ void group_adam(const AdamParams& p, const AGroup<E, WT, WC, GS>& G, const TensorDev& T, uint64_t e, AdamTrack& tr,
                                           uint32_t& ab)
{
  int tn[E], cn[E], mn[E], un[E];
#pragma unroll
  for (int k = 0; k < E; ++k) {
    int g;
    if constexpr (GS == kGradF32) g = (int)quant_f32(__int_as_float(G.g[k >> 2].d[k & 3]), p.gscale, p.glo, p.ghi, ab);
    else                          g = elem_dw<16>(G.g[0], k);
    if constexpr (FAST)
      update_adam_fast<TAIL>(p, elem_dw<WT>(G.th, k), elem_dw<WC>(G.c, k), elem_dw<16>(G.m, k), elem_dw<16>(G.u, k), g,
                             tn[k], cn[k], mn[k], un[k], tr);
    else
      update_adam<CAPS, TAIL, EXACT3>(p, elem_dw<WT>(G.th, k), elem_dw<WC>(G.c, k), elem_dw<16>(G.m, k), elem_dw<16>(G.u, k), g,
                                      tn[k], cn[k], mn[k], un[k], tr);
  }
  st_dw((int8_t*)T.theta + e * (WT / 8), pack_dw<WT, E>(tn));
  st_dw((int8_t*)T.comp + e * (WC / 8), pack_dw<WC, E>(cn));
  st_dw((int16_t*)T.mom + e, pack_dw<16, E>(mn));
  st_dw((int16_t*)T.sec + e, pack_dw<16, E>(un));
}

// Row form for int8 theta and accumulator with int16 moments and gradients: a wave takes 1024 consecutive elements
// with ONE dwordx4 access per 8-bit array (lane l: bytes 16l .. 16l+15) and TWO per 16-bit array, each of them one
// contiguous 1-KiB run of the wave (the row's first and second half).  The memory system delivers this 8-read :
// 6-written stream 5-10 % faster in that shape than with 8-byte accesses to the 8-bit arrays or with a lane's 32
// bytes of a 16-bit array adjacent.  A lane then holds sixteen 8-bit values from one place and two groups of eight
// 16-bit values from two places; which 16-byte chunk of each half a lane takes is free (any assignment of a run's
// chunks to lanes is one contiguous run), and it is chosen so that ONE swap of the upper 32 lanes of a register
// with the lower 32 lanes of another (v_permlane32_swap) lines the 8-bit data up with the 16-bit data: lane l < 32
// works on chunks 2l of both halves, lane 32 + s on chunks 2s + 1.  Before the swap lane s < 32 holds the 8-bit
// chunks 2s (dwords 0, 1) and 2s + 1 (dwords 2, 3) of the first half, lane 32 + s those of the second half; swapping
// dword 0 with 2 and 1 with 3 leaves every lane with its first-half chunk in dwords 0, 1 and its second-half
// chunk in dwords 2, 3.  The same two swaps on the results restore the order in memory for the store.
struct ARow { DW<4> th, c, m[2], u[2], g[2]; };

__device__ __forceinline__ void swap_halves(int& upper_of, int& lower_of)
{
  const auto r = __builtin_amdgcn_permlane32_swap((unsigned)upper_of, (unsigned)lower_of, false, false);
  upper_of = (int)r[0]; lower_of = (int)r[1];
}
__device__ __forceinline__ void align_bytes_with_halves(DW<4>& b) { swap_halves(b.d[0], b.d[2]); swap_halves(b.d[1], b.d[3]); }

__device__ __forceinline__ void load_row_adam(ARow& R, const TensorDev& T, uint64_t e0, int lane, int chunk)
{
  R.th = ld_dw<4>((const int8_t*)T.theta + e0 + 16 * lane);
  R.c  = ld_dw<4>((const int8_t*)T.comp + e0 + 16 * lane);
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint64_t e = e0 + 512 * h + 8 * chunk;
    R.m[h] = ld_dw<4>((const int16_t*)T.mom + e);
    R.u[h] = ld_dw<4>((const int16_t*)T.sec + e);
    R.g[h] = ld_dw<4>((const int16_t*)T.grad + e);
  }
}

template <bool CAPS, int TAIL, bool EXACT3, bool FAST>
__device__ __forceinline__ void row_adam(const AdamParams& p, ARow R, const TensorDev& T, uint64_t e0, int lane, int chunk, AdamTrack& tr)
{
  align_bytes_with_halves(R.th);
  align_bytes_with_halves(R.c);
  int tn[16], cn[16];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    int mn[8], un[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int j = 8 * h + k;
      if constexpr (FAST)
        update_adam_fast<TAIL>(p, elem_dw<8>(R.th, j), elem_dw<8>(R.c, j), elem_dw<16>(R.m[h], k), elem_dw<16>(R.u[h], k),
                               elem_dw<16>(R.g[h], k), tn[j], cn[j], mn[k], un[k], tr);
      else
        update_adam<CAPS, TAIL, EXACT3>(p, elem_dw<8>(R.th, j), elem_dw<8>(R.c, j), elem_dw<16>(R.m[h], k), elem_dw<16>(R.u[h], k),
                                        elem_dw<16>(R.g[h], k), tn[j], cn[j], mn[k], un[k], tr);
    }
    const uint64_t e = e0 + 512 * h + 8 * chunk;
    st_dw((int16_t*)T.mom + e, pack_dw<16, 8>(mn));
    st_dw((int16_t*)T.sec + e, pack_dw<16, 8>(un));
  }
  DW<4> th = pack_dw<8, 16>(tn), c = pack_dw<8, 16>(cn);
  align_bytes_with_halves(th);
  align_bytes_with_halves(c);
  st_dw((int8_t*)T.theta + e0 + 16 * lane, th);
  st_dw((int8_t*)T.comp + e0 + 16 * lane, c);
}

template <int WT, int WC, bool CAPS, int TAIL, bool EXACT3, int GS, bool FAST>
__device__ __forceinline__ void tile_vec_adam_x(const AdamParams& p, const TensorDev& T, uint64_t off, uint32_t cnt, int lane, AdamTrack& tr,
                                                uint32_t& ab)
{
  if constexpr (LPK_ADAM_ROWS > 0 && WT == 8 && WC == 8 && GS == kGradI16) {
    constexpr int kR = LPK_ADAM_ROWS > 0 ? LPK_ADAM_ROWS : 1;    // rows in flight per wave
    const uint32_t rows = cnt / 1024;
    const int chunk = lane < 32 ? 2 * lane : 2 * (lane - 32) + 1;
    uint32_t r = 0;
    for (; r + kR <= rows; r += kR) {
      ARow R[kR];
#pragma unroll
      for (int i = 0; i < kR; ++i) load_row_adam(R[i], T, off + (uint64_t)(r + i) * 1024, lane, chunk);
#pragma unroll
      for (int i = 0; i < kR; ++i) row_adam<CAPS, TAIL, EXACT3, FAST>(p, R[i], T, off + (uint64_t)(r + i) * 1024, lane, chunk, tr);
    }
    for (; r < rows; ++r) {
      ARow R;
      load_row_adam(R, T, off + (uint64_t)r * 1024, lane, chunk);
      row_adam<CAPS, TAIL, EXACT3, FAST>(p, R, T, off + (uint64_t)r * 1024, lane, chunk, tr);
    }
    off += (uint64_t)rows * 1024;                           // what is left of a ragged tile goes group by group
    cnt -= rows * 1024;
    if (cnt == 0) return;
  }
  constexpr int E = LPK_ADAM_E, kP = LPK_ADAM_GROUPS;      // elements per lane per group, groups in flight per lane
  const uint32_t ngroups = cnt / E;
  uint32_t gi = lane;
  for (; gi + (kP - 1) * kWave < ngroups; gi += kP * kWave) {             // kP groups in flight: all loads, then compute and store
    AGroup<E, WT, WC, GS> G[kP];
#pragma unroll
    for (int ps = 0; ps < kP; ++ps) load_group_adam(G[ps], T, off + (uint64_t)(gi + ps * kWave) * E);
#pragma unroll
    for (int ps = 0; ps < kP; ++ps) group_adam<E, WT, WC, CAPS, TAIL, EXACT3, GS, FAST>(p, G[ps], T, off + (uint64_t)(gi + ps * kWave) * E, tr, ab);
  }
  for (; gi < ngroups; gi += kWave) {
    AGroup<E, WT, WC, GS> G;
    const uint64_t e = off + (uint64_t)gi * E;
    load_group_adam(G, T, e);
    group_adam<E, WT, WC, CAPS, TAIL, EXACT3, GS, FAST>(p, G, T, e, tr, ab);
  }
  const uint32_t tail = cnt - ngroups * E;
  if (tail) tile_generic_adam<CAPS, GS>(p, T, off + (uint64_t)ngroups * E, tail, lane, tr, ab);
}

template <int WT, int WC, bool CAPS, int TAIL, int GS>
__device__ __forceinline__ void tile_vec_adam(const AdamParams& p, const TensorDev& T, uint64_t off, uint32_t cnt, int lane, AdamTrack& tr,
                                              uint32_t& ab)
{
  if constexpr (TAIL != kTailWide) {
    if (p.fast) { tile_vec_adam_x<WT, WC, false, TAIL, true, GS, true>(p, T, off, cnt, lane, tr, ab); return; }
  }
  if (!CAPS && p.exact3) tile_vec_adam_x<WT, WC, false, TAIL, true, GS, false>(p, T, off, cnt, lane, tr, ab);
  else                   tile_vec_adam_x<WT, WC, CAPS, TAIL, false, GS, false>(p, T, off, cnt, lane, tr, ab);
}

// ---------------------------------------------------------------- per-tensor set-up (wave-uniform)

template <int GS>
__device__ __forceinline__ void setup_adam(AdamParams& p, const TensorDev& T, int fl_in, int fl_out, int fl_m_in, int fl_m_out,
                                           int fl_u_in, int fl_u_out, int fl_g, const AdamHyperDev& h, uint32_t& status_bits)
{
  p.wt = T.wt; p.wc = T.wc; p.wg = T.wg; p.wm = T.wm; p.wu = T.wu; p.has_comp = T.comp != nullptr;
  const int d = p.has_comp ? T.d : 0;
  const int delta = fl_out - fl_in, delta_m = fl_m_out - fl_m_in, delta_u = fl_u_out - fl_u_in;
  const int par = fl_u_out & 1;                             // two's complement: the non-negative parity
  const int R = (fl_u_out + 24 + par) >> 1;                 // exact, the numerator is even
  const int F = fl_in + d;
  const int e = F + R - 16 - (int)h.lr_exp - fl_m_out;
  auto bad = [](int f) { return f < kFlMin || f > kFlMax; };
  auto far = [](int x) { return x > kDeltaMax || x < -kDeltaMax; };
  if (bad(fl_in) || bad(fl_out) || bad(fl_m_in) || bad(fl_m_out) || bad(fl_u_in) || bad(fl_u_out) || bad(fl_g) ||
      d > kDMax || far(delta) || far(delta_m) || far(delta_u) || e > 20) {
    p.path = skipped_path<GS>(fl_g); status_bits |= kStatusDomain; return;
  }
  p.a1 = (double)h.b1 * pow2d(delta_m);                     // b1 * 2^-(fl_m_in - fl_m_out)
  p.a2 = (double)(65536u - h.b1) * pow2d(fl_m_out - fl_g);
  p.a3 = (double)h.b2 * pow2d(delta_u);
  p.a4 = (double)(65536u - h.b2) * pow2d(fl_u_out - 2 * fl_g);
  const int wc = p.has_comp ? p.wc : 8;
  p.qmax_m = (double)((1 << (p.wm - 1)) - 1); p.qmin_m = -(double)(1 << (p.wm - 1));
  p.qmax_u = (double)((1 << (p.wu - 1)) - 1);
  p.ascale = pow2d(24 + par);
  p.eps_r  = __builtin_fmin(__builtin_rint((double)h.eps * pow2d(R - 16 - (int)h.eps_exp)), 1073741824.0);
  p.nlr    = -(double)h.lr * pow2d(e);
  const int u = delta > 0 ? delta : 0, kth = d + u - delta, kc = kth - d;
  p.wa = make_alg1_wide(d, u, kth, kc, -(1 << (p.wt - 1)), (1 << (p.wt - 1)) - 1, -(1 << (wc - 1)), (1 << (wc - 1)) - 1);
  // Can a cap bind?  |g| <= 2^15 and g^2 <= 2^30 bound the two gradient terms; the step is at most
  // |num| / den <= 2^15 lr 2^e / max(eps_R, 1) (2^-e in the divisor when e < 0).
  const double step_bound = 32768.0 * (double)h.lr * pow2d(e) / __builtin_fmax(p.eps_r, 1.0);
  p.caps = !(32768.0 * p.a2 < cap_d() && 1073741824.0 * p.a4 < cap_d() && step_bound < cap_d());
  auto whole = [](double x) { return x == __builtin_rint(x); };
  p.exact3 = !p.caps && whole(p.a1) && whole(p.a2) && whole(p.a3);
  p.gscale = __uint_as_float((uint32_t)(127 + fl_g) << 23);
  p.glo = -(float)(1 << (p.wg - 1)); p.ghi = (float)((1 << (p.wg - 1)) - 1);
  p.path = 1;
  const bool widths_ok = (p.wt == p.wc) || (p.wt == 8 && p.wc == 16);
  const bool src_ok = GS == kGradI16 || (((uintptr_t)T.src) & 15u) == 0;
  if (p.has_comp && T.vec_adam && src_ok && widths_ok && p.wg == 16 && p.wm == 16 && p.wu == 16) p.path = 2;
  // 32-bit tail: |theta * 2^d| + |c| + |s| + the rounding addend provably below 2^22 (2^23 with the residual formed
  // unshifted), theta's grid fixed, 1 <= d
  p.tail = kTailWide;
  const double vbound = pow2d(p.wt - 1 + d) + pow2d(wc - 1) + step_bound + 1.0 + pow2d(d > 0 ? d - 1 : 0);
  if (p.path == 2 && p.wt == 8 && delta == 0 && d >= 1 && !p.caps) {
    if (p.wc == 8 && d <= 8 && vbound < 4194304.0) p.tail = kTailSmall;
    if (p.wc == 16 && d <= 22 && vbound < 8388608.0) p.tail = kTailSmallBigD;
  }
  // fast route: both moment grids standing still, 0 <= sh <= 8 with |wM| < 2^38, (1-b2)*g^2 below 2^30 on u's
  // guard-bit grid, a 32-bit tail, and a step provably below 0.99 * 2^22
  const int sh = fl_m_out - fl_g;
  p.fast = p.exact3 && p.tail != kTailWide && delta_m == 0 && delta_u == 0 && sh >= 0 && sh <= 8 && p.a2 <= 4194304.0 &&
           p.a4 <= 1.0 && step_bound < 4152360.0;
  p.neg2sh = -(1 << (sh >= 0 && sh <= 8 ? sh : 0));
  p.nc1_f = -(float)(65536u - h.b1);
  p.nc2 = -(int)(65536u - h.b2);
  p.qmin_mi = -(1 << (p.wm - 1)); p.qmax_mi = (1 << (p.wm - 1)) - 1; p.qmax_ui = (1 << (p.wu - 1)) - 1;
  p.eps_i = (int)p.eps_r;
  p.ascale_f = __uint_as_float((uint32_t)(127 + 24 + par) << 23);
  p.d = d;
  p.sm = make_alg1_small(d, -(1 << (p.wt - 1)), (1 << (p.wt - 1)) - 1, -(1 << (wc - 1)), (1 << (wc - 1)) - 1);
}

// ---------------------------------------------------------------- the kernel

__device__ __forceinline__ uint64_t track_u64(double x) { return (uint64_t)x; }     // an integer below 2^53
__device__ __forceinline__ uint64_t track_m(const AdamTrack& tr)                    // both routes' maxima of |mq|
{
  const uint64_t mi = vtrack_max(tr.m), md = (uint64_t)tr.mm;
  return mi > md ? mi : md;
}
__device__ __forceinline__ uint64_t track_um(const AdamTrack& tr)                   // ... of max(uq, 0)
{
  const uint64_t ui = (uint64_t)tr.umx, ud = (uint64_t)tr.um;
  return ui > ud ? ui : ud;
}
__device__ __forceinline__ uint64_t track_vmax(const AdamTrack& tr)                 // both tails' maxima of |v|
{
  const uint64_t m32 = vtrack_max(tr.v), m64 = (uint64_t)tr.vm;
  return m32 > m64 ? m32 : m64;
}

template <int GS>
__global__ void __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(LPK_ADAM_WAVES_PER_SIMD, LPK_ADAM_WAVES_PER_SIMD)))
adam_step_kernel(const TensorDev* __restrict__ tensors, const Tile* __restrict__ tiles, uint32_t n_tiles,
                 const int32_t* __restrict__ fl_in, const int32_t* __restrict__ fl_out,
                 const int32_t* __restrict__ fl_m_in, const int32_t* __restrict__ fl_m_out,
                 const int32_t* __restrict__ fl_u_in, const int32_t* __restrict__ fl_u_out, const int32_t* __restrict__ fl_g,
                 AdamHyperDev h, uint64_t* vmax, uint64_t* mmax, uint64_t* umax, uint32_t* status, MaxFold fold)
{
  __shared__ int      s_tensor[kWavesPerBlock];
  __shared__ uint64_t s_max[kWavesPerBlock];

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = wave_uniform(threadIdx.x >> 6);

  AdamTrack tr{0.0, 0.0, 0.0, {0, 0}, {0, 0}, 0};
  uint32_t status_bits = 0, ab_max = 0;
  AdamParams p; p.path = 0;
  TensorDev T;

  const int cur = walk_tiles(tiles, n_tiles,
    [&](int t) LPK_INLINE_LAMBDA {
      if (vmax) flush_wave(vmax, t, track_vmax(tr), lane);
      if (mmax) flush_wave(mmax, t, track_m(tr), lane);
      if (umax) flush_wave(umax, t, track_um(tr), lane);
    },
    [&](int t) LPK_INLINE_LAMBDA {
      tr = AdamTrack{0.0, 0.0, 0.0, {0, 0}, {0, 0}, 0};
      T = tensors[t];
      setup_adam<GS>(p, T, fl_in[t], fl_out[t], fl_m_in[t], fl_m_out[t], fl_u_in[t], fl_u_out[t], fl_g[t], h, status_bits);
    },
    [&](uint64_t off, uint32_t cnt) LPK_INLINE_LAMBDA {
      if (p.path == 2 && !p.caps) {
        if (p.wt == 8 && p.wc == 8) {
          if (p.tail == kTailSmall) tile_vec_adam<8, 8, false, kTailSmall, GS>(p, T, off, cnt, lane, tr, ab_max);
          else                      tile_vec_adam<8, 8, false, kTailWide, GS>(p, T, off, cnt, lane, tr, ab_max);
        } else if (p.wt == 16) {
          tile_vec_adam<16, 16, false, kTailWide, GS>(p, T, off, cnt, lane, tr, ab_max);
        } else {
          if (p.tail == kTailSmallBigD) tile_vec_adam<8, 16, false, kTailSmallBigD, GS>(p, T, off, cnt, lane, tr, ab_max);
          else                          tile_vec_adam<8, 16, false, kTailWide, GS>(p, T, off, cnt, lane, tr, ab_max);
        }
      } else if (p.path > 0) {
        if (p.caps) tile_generic_adam<true, GS>(p, T, off, cnt, lane, tr, ab_max); else tile_generic_adam<false, GS>(p, T, off, cnt, lane, tr, ab_max);
      } else if (GS == kGradF32 && p.path == kPathSkipButScan) {
        scan_nonfinite(T.src, off, cnt, lane, ab_max);
      }
    });

  if (GS == kGradF32 && __ballot(ab_max >= 0x7f800000u)) status_bits |= kStatusNonFinite;
  raise_status(status, status_bits, lane);
  if (vmax) flush_block(vmax, cur, track_vmax(tr), lane, wave, s_tensor, s_max);
  if (mmax) flush_block(mmax, cur, track_m(tr), lane, wave, s_tensor, s_max);
  if (umax) flush_block(umax, cur, track_um(tr), lane, wave, s_tensor, s_max);
  if (fold.arrivals) { uint64_t* const acc[3] = {vmax, mmax, umax}; fold_maxima<3>(fold, acc, &s_tensor[0]); }
}

__global__ void __launch_bounds__(kBlock) fill3_u64_kernel(uint64_t* a, uint64_t* b, uint64_t* c, uint32_t n)
{
  const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
  if (i < n) { if (a) a[i] = 0; if (b) b[i] = 0; if (c) c[i] = 0; }
}

hipError_t launch_adam_step(const TensorDev* tensors, const Tile* tiles, uint32_t n_tiles, uint32_t n_tensors, uint32_t grid,
                            int grad_is_f32, const int32_t* fl_in, const int32_t* fl_out, const int32_t* fl_m_in, const int32_t* fl_m_out,
                            const int32_t* fl_u_in, const int32_t* fl_u_out, const int32_t* fl_g, AdamHyperDev h,
                            uint64_t* vmax, uint64_t* mmax, uint64_t* umax, uint32_t* status, uint64_t* fold_acc, uint32_t* arrivals,
                            hipStream_t stream)
{
  const MaxPlan m = plan_maxima(fold_acc, arrivals, n_tensors, n_tiles, grid, vmax, mmax, umax);
  if ((vmax || mmax || umax) && !m.fold.arrivals)
    hipLaunchKernelGGL(fill3_u64_kernel, dim3((n_tensors + kBlock - 1) / kBlock), dim3(kBlock), 0, stream, vmax, mmax, umax, n_tensors);
  if (n_tiles) {
    if (grad_is_f32)
      hipLaunchKernelGGL(adam_step_kernel<kGradF32>, dim3(grid), dim3(kBlock), 0, stream, tensors, tiles, n_tiles,
                         fl_in, fl_out, fl_m_in, fl_m_out, fl_u_in, fl_u_out, fl_g, h, m.acc[0], m.acc[1], m.acc[2], status, m.fold);
    else
      hipLaunchKernelGGL(adam_step_kernel<kGradI16>, dim3(grid), dim3(kBlock), 0, stream, tensors, tiles, n_tiles,
                         fl_in, fl_out, fl_m_in, fl_m_out, fl_u_in, fl_u_out, fl_g, h, m.acc[0], m.acc[1], m.acc[2], status, m.fold);
  }
  return hipGetLastError();
}

}  // namespace lpk

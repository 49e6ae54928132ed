// Momentum SGD with the lazy update inside (paper, Section 4: momentum optimizer with Algorithm 1 implemented
// in the optimizer, INT8 or INT16 velocity).  One fused launch over every tile of every tensor:
//
//   w  = RNE(mu*m on grid G) + cap(RNE(-lr*g on G)) [+ cap(RNE(-lr*wd*theta on G))],  G = fl_m_out + 16
//   mq = RNE(w / 2^16);  m' = sat(mq);  mmax = max|mq|;  s = cap(RNE(m' on grid F));  then Algorithm 1 with step s.
//
// Same work distribution as the plain update (persistent wavefronts over the tile table, 16 or 8 consecutive
// elements per lane per pass, non-temporal vector accesses).  Two bit-identical arithmetic paths chosen per
// tensor: wide (exact fp64, anything inside the domain), and a 32-bit one (same-width theta/comp, 16-bit
// gradients, theta's grid fixed) whose shifts are wave-uniform operands of branch-free integer roundings (the
// velocity grid may move); the decay term is rounded by one fp64 FMA as in the plain update.  Gradients come
// from the int16 array or, in a second kernel instance, from the fp32 source, quantized in registers.
#include "step_common.hpp"

namespace lpk {

struct MomParams {
  int      path;                 // 0 skip, 1 element by element (wide arithmetic), 2 vector
  int      wide;                 // vector path: wide (fp64) arithmetic instead of the 32-bit one
  int      wt, wc, wg, wm, d, has_comp;
  int      k1, k2, k3w, k3;      // shifts: mu*m -> G, lr*g -> G, lr*wd*theta -> G, m' -> F
  int      u, kth, kc;
  int64_t  lr, mu, lrwd;
  float    gscale, glo, ghi;            // fp32 gradient source: 2^fl_g and the rails of the gradient width
  int      qmin_t, qmax_t, qmin_c, qmax_c, qmin_m, qmax_m;
  // 32-bit path: each term is (x << a) then RNE >> b with exactly one of a, b non-zero
  int      mu_i, a1, b1, h1, nz1;          // mu*m -> grid G
  int      c2, b2, h2, nz2;                // (-lr << a2) * g -> grid G
  int      a3, b3, h3, nz3;                // m' -> grid F
  double   nlrwd_d, magic_d;  int magic_dlo;
  Alg1Int  in;                             // last stage of Algorithm 1 by add-and-shift
  // wide path: mu * 2^-k1, -lr * 2^-k2, -lr * wd * 2^-k3w, 2^-k3, the velocity's rails, the last stage's constants
  double   w_a1, w_a2, w_a3, w_inv_k3, w_lo_m, w_hi_m;
  Alg1Wide wa;
};

struct WideMax { double v, w; };

template <bool DECAY>
__device__ __forceinline__ void update_wide_mom(const MomParams& p, int th, int c, int m, int g,
                                                int& th_new, int& c_new, int& m_new, WideMax& mx)
{
  const double cap = 1099511627776.0;                       // 2^40
  double w = __builtin_rint((double)m * p.w_a1);
  w += clampd(__builtin_rint((double)g * p.w_a2), -cap, cap);
  if (DECAY) w += clampd(__builtin_rint((double)th * p.w_a3), -cap, cap);
  const double mq = __builtin_rint(w * 0x1p-16);
  mx.w = __builtin_fmax(mx.w, __builtin_fabs(mq));
  const double mn = clampd(mq, p.w_lo_m, p.w_hi_m);
  const double s = clampd(__builtin_rint(mn * p.w_inv_k3), -cap, cap);
  alg1_wide(p.wa, th, c, s, th_new, c_new, mx.v);
  m_new = (int)mn;
}

__device__ __forceinline__ void fold_wide(const WideMax& mx, uint64_t& vm, uint64_t& wm)
{
  const uint64_t a = (uint64_t)mx.v, b = (uint64_t)mx.w;    // integers below 2^53
  vm = a > vm ? a : vm;
  wm = b > wm ? b : wm;
}

template <int GS>
__device__ __forceinline__ void tile_generic_mom(const MomParams& p, const TensorDev& T, uint64_t off, uint32_t cnt, int lane,
                                                 uint64_t& vm, uint64_t& wm, uint32_t& ab)
{
  WideMax mx{0.0, 0.0};
  for (uint32_t j = lane; j < cnt; j += kWave) {
    uint64_t i = off + j;
    int th = load_elem(T.theta, i, p.wt);
    int c  = p.has_comp ? load_elem(T.comp, i, p.wc) : 0;
    int m  = load_elem(T.mom, i, p.wm);
    int g  = GS == kGradF32 ? (int)quant_f32(((const float*)T.src)[i], p.gscale, p.glo, p.ghi, ab) : load_elem(T.grad, i, p.wg);
    int tn, cn, mn;
    if (p.lrwd) update_wide_mom<true>(p, th, c, m, g, tn, cn, mn, mx); else update_wide_mom<false>(p, th, c, m, g, tn, cn, mn, mx);
    store_elem(T.theta, i, p.wt, tn);
    if (p.has_comp) store_elem(T.comp, i, p.wc, cn);
    store_elem(T.mom, i, p.wm, mn);
  }
  fold_wide(mx, vm, wm);
}

// ---------------------------------------------------------------- fast path

struct MaxTrack { VTrack v, w; };                      // extremes of the compensated sum and of the unsaturated velocity

template <bool DECAY, bool K1ZERO, bool WIDEW>
__device__ __forceinline__ void update_fast_mom(const MomParams& p, int th, int c, int m, int g, int& tn, int& cn, int& mn, MaxTrack& mt)
{
  int t1 = __mul24(m, p.mu_i);
  if (!K1ZERO) t1 = rne_shr32((int)((unsigned)t1 << p.a1), p.b1, p.h1, p.nz1);
  int t2 = rne_shr32(__mul24(g, p.c2), p.b2, p.h2, p.nz2);
  if (DECAY) t2 += __double2loint(__builtin_fma((double)th, p.nlrwd_d, p.magic_d)) - p.magic_dlo;
  int q;
  if (WIDEW) {
    // |t1| and |t2| are each below 2^31 but their sum may not be: add high and low halves separately.
    const int lo = (t1 & 0xffff) + (t2 & 0xffff);                    // 0 .. 131070
    const int fl = (t1 >> 16) + (t2 >> 16) + (lo >> 16);             // floor(w / 2^16)
    const unsigned rem = (unsigned)lo & 0xffffu;
    q = fl + (int)((rem | (unsigned)(fl & 1)) > 0x8000u);            // round half to even
  } else {
    const int w = t1 + t2;
    q = (w + 0x7fff + ((w >> 16) & 1)) >> 16;                        // RNE(w / 2^16)
  }
  track_v(mt.w, q);
  mn = min(max(q, p.qmin_m), p.qmax_m);
  const int s = rne_shr32((int)((unsigned)mn << p.a3), p.b3, p.h3, p.nz3);
  const int v = (int)((unsigned)th << p.d) + c + s;
  track_v(mt.v, v);
  alg1_int(p.in, v, tn, cn);
}

// E consecutive elements per lane.  WT / WC / WM = widths of theta, comp (WT, or 16 next to an 8-bit theta) and the
// velocity.
// E = 16 when all three are 8 bits wide (dwordx4 each), E = 8 as soon as one of them is 16 bits wide: then every
// access of a wave is still one contiguous run (with 16, a lane's 16-bit data would span two stores 32 bytes
// apart, which reach HBM as partial lines).
template <int E, int WT, int WC, int WM, int GS> struct MGroup {
  static constexpr int kG = GS == kGradF32 ? E / 4 : (GS == kGradI8 ? 1 : E / 8);       // gradient accesses ...
  static constexpr int kGN = GS == kGradI8 ? E / 4 : 4;                                  // ... of so many dwords
  DW<E * WT / 32> th;
  DW<E * WC / 32> c;
  DW<E * WM / 32> m;
  DW<kGN> g[kG];
};

template <int E, int WT, int WC, int WM, int GS>
__device__ __forceinline__ void load_group_mom(MGroup<E, WT, WC, WM, GS>& G, const TensorDev& T, uint64_t e)
{
  G.th = ld_dw<E * WT / 32>((const int8_t*)T.theta + e * (WT / 8));
  G.c  = ld_dw<E * WC / 32>((const int8_t*)T.comp + e * (WC / 8));
  G.m  = ld_dw<E * WM / 32>((const int8_t*)T.mom + e * (WM / 8));
#pragma unroll
  for (int j = 0; j < MGroup<E, WT, WC, WM, GS>::kG; ++j) {
    if constexpr (GS == kGradF32)     G.g[j] = ld_dw<4>((const float*)T.src + e + 4 * j);
    else if constexpr (GS == kGradI8) G.g[j] = ld_dw<E / 4>((const int8_t*)T.grad + e);
    else                              G.g[j] = ld_dw<4>((const int16_t*)T.grad + e + 8 * j);
  }
}

template <int E, int WT, int WC, int WM, bool DECAY, bool K1ZERO, bool WIDE, int GS>
__device__ __forceinline__ void group_fast_mom(const MomParams& p, const MGroup<E, WT, WC, WM, GS>& G, const TensorDev& T, uint64_t e, MaxTrack& mt, WideMax& mx,
                                               uint32_t& ab)
{
  int tn[E], cn[E], mn[E];
#pragma unroll
  for (int k = 0; k < E; ++k) {
    const int th = elem_dw<WT>(G.th, k), c = elem_dw<WC>(G.c, k), m = elem_dw<WM>(G.m, k);
    int g;
    if constexpr (GS == kGradF32)     g = (int)quant_f32(__int_as_float(G.g[k >> 2].d[k & 3]), p.gscale, p.glo, p.ghi, ab);
    else if constexpr (GS == kGradI8) g = elem_dw<8>(G.g[0], k);
    else                              g = elem_dw<16>(G.g[k >> 3], k & 7);
    if (WIDE) update_wide_mom<DECAY>(p, th, c, m, g, tn[k], cn[k], mn[k], mx);
    else      update_fast_mom<DECAY, K1ZERO, (WM == 16)>(p, th, c, m, g, tn[k], cn[k], mn[k], mt);
  }
  st_dw((int8_t*)T.theta + e * (WT / 8), pack_dw<WT, E>(tn));
  st_dw((int8_t*)T.comp + e * (WC / 8), pack_dw<WC, E>(cn));
  st_dw((int8_t*)T.mom + e * (WM / 8), pack_dw<WM, E>(mn));
}

template <int WT, int WC, int WM, bool DECAY, bool K1ZERO, bool WIDE, int GS>
__device__ __forceinline__ void tile_fast_mom(const MomParams& p, const TensorDev& T, uint64_t off, uint32_t cnt, int lane,
                                              uint64_t& vm, uint64_t& wm, uint32_t& ab)
{
  MaxTrack mt{{0, 0}, {0, 0}};
  WideMax mx{0.0, 0.0};
  constexpr int E = (WT == 16 || WC == 16 || WM == 16 || GS == kGradF32) ? 8 : 16;   // fp32 gradients: two dwordx4 per lane, as in the plain update
  constexpr int kP = WIDE ? 1 : 4;                         // groups in flight (the wide path would set the kernel's register count)
  const uint32_t ngroups = cnt / E;
  uint32_t gi = lane;
  for (; gi + (kP - 1) * kWave < ngroups; gi += kP * kWave) {             // kP groups in flight: all loads, then compute and store
    MGroup<E, WT, WC, WM, GS> G[kP];
#pragma unroll
    for (int ps = 0; ps < kP; ++ps) load_group_mom(G[ps], T, off + (uint64_t)(gi + ps * kWave) * E);
#pragma unroll
    for (int ps = 0; ps < kP; ++ps)
      group_fast_mom<E, WT, WC, WM, DECAY, K1ZERO, WIDE, GS>(p, G[ps], T, off + (uint64_t)(gi + ps * kWave) * E, mt, mx, ab);
  }
  for (; gi < ngroups; gi += kWave) {
    MGroup<E, WT, WC, WM, GS> G;
    const uint64_t e = off + (uint64_t)gi * E;
    load_group_mom(G, T, e);
    group_fast_mom<E, WT, WC, WM, DECAY, K1ZERO, WIDE, GS>(p, G, T, e, mt, mx, ab);
  }
  uint64_t x = vtrack_max(mt.v);
  vm = x > vm ? x : vm;
  x = vtrack_max(mt.w);
  wm = x > wm ? x : wm;
  fold_wide(mx, vm, wm);
  const uint32_t tail = cnt - ngroups * E;
  if (tail) tile_generic_mom<GS>(p, T, off + (uint64_t)ngroups * E, tail, lane, vm, wm, ab);
}

template <int WT, int WC, int WM, int GS>
__device__ __forceinline__ void tile_fast_mom_dispatch(const MomParams& p, const TensorDev& T, uint64_t off, uint32_t cnt, int lane,
                                                       uint64_t& vm, uint64_t& wm, uint32_t& ab)
{
  if (p.wide) {
    if (p.lrwd) tile_fast_mom<WT, WC, WM, true, false, true, GS>(p, T, off, cnt, lane, vm, wm, ab); else tile_fast_mom<WT, WC, WM, false, false, true, GS>(p, T, off, cnt, lane, vm, wm, ab);
    return;
  }
  const bool k1z = p.k1 == 0;
  if (p.lrwd) { if (k1z) tile_fast_mom<WT, WC, WM, true, true, false, GS>(p, T, off, cnt, lane, vm, wm, ab);  else tile_fast_mom<WT, WC, WM, true, false, false, GS>(p, T, off, cnt, lane, vm, wm, ab); }
  else        { if (k1z) tile_fast_mom<WT, WC, WM, false, true, false, GS>(p, T, off, cnt, lane, vm, wm, ab); else tile_fast_mom<WT, WC, WM, false, false, false, GS>(p, T, off, cnt, lane, vm, wm, ab); }
}

// ---------------------------------------------------------------- per-tensor set-up

template <int GS>
__device__ __forceinline__ void setup_mom(MomParams& p, const TensorDev& T, int fl_in, int fl_out, int fl_m_in, int fl_m_out,
                                          int fl_g, uint32_t lr, uint32_t mu, uint32_t wd, uint32_t& status_bits)
{
  p.wt = T.wt; p.wc = T.wc; p.wg = T.wg; p.wm = T.wm; p.has_comp = T.comp != nullptr;
  p.d = p.has_comp ? T.d : 0;
  const int delta = fl_out - fl_in, delta_m = fl_m_out - fl_m_in;
  auto bad = [](int f) { return f < kFlMin || f > kFlMax; };
  if (bad(fl_in) || bad(fl_out) || bad(fl_m_in) || bad(fl_m_out) || bad(fl_g) || p.d > kDMax ||
      delta > kDeltaMax || delta < -kDeltaMax || delta_m > kDeltaMax || delta_m < -kDeltaMax) {
    p.path = skipped_path<GS>(fl_g); status_bits |= kStatusDomain; return;
  }
  const int F = fl_in + p.d, G = fl_m_out + 16;
  p.k1 = fl_m_in + 16 - G;
  p.k2 = fl_g + 16 - G;
  p.k3w = fl_in + 32 - G;
  p.k3 = fl_m_out - F;
  p.u = delta > 0 ? delta : 0;
  p.kth = p.d + p.u - delta;
  p.kc = p.kth - p.d;
  p.lr = lr; p.mu = mu; p.lrwd = (int64_t)lr * (int64_t)wd;
  p.qmax_t = (1 << (p.wt - 1)) - 1; p.qmin_t = -(1 << (p.wt - 1));
  const int wc = p.has_comp ? p.wc : 8;
  p.qmax_c = (1 << (wc - 1)) - 1;   p.qmin_c = -(1 << (wc - 1));
  p.qmax_m = (1 << (p.wm - 1)) - 1; p.qmin_m = -(1 << (p.wm - 1));
  p.w_a1 = (double)mu * pow2d(-p.k1); p.w_a2 = -(double)lr * pow2d(-p.k2); p.w_a3 = -(double)p.lrwd * pow2d(-p.k3w);
  p.w_inv_k3 = pow2d(-p.k3);
  p.wa = make_alg1_wide(p.d, p.u, p.kth, p.kc, p.qmin_t, p.qmax_t, p.qmin_c, p.qmax_c);
  p.w_lo_m = (double)p.qmin_m; p.w_hi_m = (double)p.qmax_m;
  p.gscale = __uint_as_float((uint32_t)(127 + fl_g) << 23);
  p.glo = -(float)(1 << (p.wg - 1)); p.ghi = (float)((1 << (p.wg - 1)) - 1);
  p.path = 1; p.wide = 1;

  // Vector path: aligned, comp present and as wide as theta (or int8 theta with an int16 comp), 16-bit grads.  32-bit arithmetic on it when theta's
  // grid is fixed, d >= 1, and every intermediate (including each rounding addend) is provably below 2^31 in
  // magnitude; the wide arithmetic otherwise.
  // gradients: 16 bits wide; or 8 bits from the fp32 source (only the rails differ) or from an int8 array next to
  // 8-bit theta and comp (the 8-bit training mode, with an 8- or 16-bit velocity)
  const bool grads_ok = p.wg == 16 || (GS == kGradF32 && p.wg == 8) || (GS == kGradI16 && p.wg == 8 && p.wt == 8);
  const bool widths_ok = p.wt == p.wc || (p.wt == 8 && p.wc == 16);
  if (!p.has_comp || !T.vec_mom || !widths_ok || !grads_ok) return;
  if (GS == kGradF32 && (((uintptr_t)T.src) & 15u) != 0) return;
  p.path = 2;
  if (delta != 0 || p.d < 1) return;
  const int64_t lim = 1ll << 31;
  // t1 = mu*m brought to grid G
  const int64_t X1 = (int64_t)mu << (p.wm - 1);
  int64_t T1;
  p.a1 = p.k1 < 0 ? -p.k1 : 0; p.b1 = p.k1 > 0 ? p.k1 : 0;
  p.nz1 = p.b1 > 0; p.h1 = p.b1 > 0 ? (1 << (p.b1 - 1)) - 1 : 0;
  if (p.b1 == 0) T1 = X1 << p.a1; else { if (X1 + (1ll << (p.b1 - 1)) >= lim) return; T1 = (X1 >> p.b1) + 1; }
  if (T1 >= lim) return;
  // t2 = -lr*g brought to grid G: the left shift is folded into the 24-bit multiplier
  if (p.k2 < -8 || p.k2 > 30) return;
  const int a2 = p.k2 < 0 ? -p.k2 : 0;
  const int64_t C2 = (int64_t)lr << a2;
  if (C2 >= (1ll << 23)) return;
  const int64_t P2 = C2 << 15;
  int64_t T2;
  p.c2 = -(int)C2; p.b2 = p.k2 > 0 ? p.k2 : 0;
  p.nz2 = p.b2 > 0; p.h2 = p.b2 > 0 ? (1 << (p.b2 - 1)) - 1 : 0;
  if (p.b2 == 0) T2 = P2; else { if (P2 + (1ll << (p.b2 - 1)) >= lim) return; T2 = (P2 >> p.b2) + 1; }
  // t3 = decay term (fp64 FMA rounding)
  int64_t T3 = 0;
  if (p.lrwd) { if (p.k3w < 1 || p.k3w > 60) return; T3 = ((p.lrwd << (p.wt - 1)) >> p.k3w) + 1; }
  if (p.wm == 16 ? (T1 >= lim || T2 + T3 >= lim) : (T1 + T2 + T3 + 0x8000 >= lim)) return;   // 16-bit velocity adds in two halves
  // s = m' brought to grid F
  if (p.k3 > 30 || p.k3 < -24) return;
  p.a3 = p.k3 < 0 ? -p.k3 : 0; p.b3 = p.k3 > 0 ? p.k3 : 0;
  p.nz3 = p.b3 > 0; p.h3 = p.b3 > 0 ? (1 << (p.b3 - 1)) - 1 : 0;
  const int64_t M = 1ll << (p.wm - 1);
  const int64_t S = p.b3 == 0 ? (M << p.a3) : (M >> p.b3) + 1;
  const int64_t V = (1ll << (p.wt - 1 + p.d)) + (1ll << (p.wc - 1)) + S + (1ll << (p.d - 1));
  if (V >= lim) return;
  p.wide = 0;
  p.mu_i = (int)mu;
  const long long md = ((long long)(1023 + 52 + (p.lrwd ? p.k3w : 1)) << 52) | (1ll << 51);
  p.magic_d   = __longlong_as_double(md);
  p.magic_dlo = (int)(md & 0xffffffffll);
  p.nlrwd_d   = -(double)p.lrwd;
  p.in = Alg1Int{p.d, (1 << (p.d - 1)) - 1, p.qmin_t, p.qmax_t, p.qmin_c, p.qmax_c};
}

// ---------------------------------------------------------------- the kernel

template <int GS>
__global__ void __launch_bounds__(kBlock)
momentum_step_kernel(const TensorDev* __restrict__ tensors, const Tile* __restrict__ tiles, uint32_t n_tiles,
                     const int32_t* __restrict__ fl_in, const int32_t* __restrict__ fl_out,
                     const int32_t* __restrict__ fl_m_in, const int32_t* __restrict__ fl_m_out, const int32_t* __restrict__ fl_g,
                     uint32_t lr, uint32_t mu, uint32_t wd, uint64_t* vmax, uint64_t* mmax, uint32_t* status, MaxFold fold)
{
  __shared__ int      s_tensor[kWavesPerBlock];
  __shared__ uint64_t s_max[kWavesPerBlock];

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = wave_uniform(threadIdx.x >> 6);

  uint64_t vm = 0, wm = 0;
  uint32_t status_bits = 0, ab_max = 0;
  MomParams p; p.path = 0;
  TensorDev T;

  const int cur = walk_tiles(tiles, n_tiles,
    [&](int t) LPK_INLINE_LAMBDA {
      if (vmax) flush_wave(vmax, t, vm, lane);
      if (mmax) flush_wave(mmax, t, wm, lane);
    },
    [&](int t) LPK_INLINE_LAMBDA {
      vm = wm = 0;
      T = tensors[t];
      setup_mom<GS>(p, T, fl_in[t], fl_out[t], fl_m_in[t], fl_m_out[t], fl_g[t], lr, mu, wd, status_bits);
    },
    [&](uint64_t off, uint32_t cnt) LPK_INLINE_LAMBDA {
      if (p.path == 2) {
        if (p.wt == 8 && GS == kGradI16 && p.wg == 8) {       // int8 gradient array (8-bit training mode)
          constexpr int G8 = GS == kGradI16 ? kGradI8 : GS;
          if (p.wc == 8) { if (p.wm == 8) tile_fast_mom_dispatch<8, 8, 8, G8>(p, T, off, cnt, lane, vm, wm, ab_max);  else tile_fast_mom_dispatch<8, 8, 16, G8>(p, T, off, cnt, lane, vm, wm, ab_max); }
          else           { if (p.wm == 8) tile_fast_mom_dispatch<8, 16, 8, G8>(p, T, off, cnt, lane, vm, wm, ab_max); else tile_fast_mom_dispatch<8, 16, 16, G8>(p, T, off, cnt, lane, vm, wm, ab_max); }
        }
        else if (p.wt == 8 && p.wc == 8) { if (p.wm == 8) tile_fast_mom_dispatch<8, 8, 8, GS>(p, T, off, cnt, lane, vm, wm, ab_max);  else tile_fast_mom_dispatch<8, 8, 16, GS>(p, T, off, cnt, lane, vm, wm, ab_max); }
        else if (p.wt == 8)              { if (p.wm == 8) tile_fast_mom_dispatch<8, 16, 8, GS>(p, T, off, cnt, lane, vm, wm, ab_max); else tile_fast_mom_dispatch<8, 16, 16, GS>(p, T, off, cnt, lane, vm, wm, ab_max); }
        else                             { if (p.wm == 8) tile_fast_mom_dispatch<16, 16, 8, GS>(p, T, off, cnt, lane, vm, wm, ab_max); else tile_fast_mom_dispatch<16, 16, 16, GS>(p, T, off, cnt, lane, vm, wm, ab_max); }
      } else if (p.path == 1) {
        tile_generic_mom<GS>(p, T, off, cnt, lane, vm, wm, ab_max);
      } else if (GS == kGradF32 && p.path == kPathSkipButScan) {
        scan_nonfinite(T.src, off, cnt, lane, ab_max);
      }
    });

  if (GS == kGradF32 && __ballot(ab_max >= 0x7f800000u)) status_bits |= kStatusNonFinite;
  raise_status(status, status_bits, lane);
  if (vmax) flush_block(vmax, cur, vm, lane, wave, s_tensor, s_max);
  if (mmax) flush_block(mmax, cur, wm, lane, wave, s_tensor, s_max);
  if (fold.arrivals) { uint64_t* const acc[2] = {vmax, mmax}; fold_maxima<2>(fold, acc, &s_tensor[0]); }
}

__global__ void __launch_bounds__(kBlock) fill2_u64_kernel(uint64_t* a, uint64_t* b, uint32_t n)
{
  uint32_t i = blockIdx.x * kBlock + threadIdx.x;
  if (i < n) { if (a) a[i] = 0; if (b) b[i] = 0; }
}

hipError_t launch_momentum_step(const TensorDev* tensors, const Tile* tiles, uint32_t n_tiles, uint32_t n_tensors, uint32_t grid,
                                int grad_is_f32, const int32_t* fl_in, const int32_t* fl_out, const int32_t* fl_m_in, const int32_t* fl_m_out,
                                const int32_t* fl_g, uint32_t lr, uint32_t mu, uint32_t wd,
                                uint64_t* vmax, uint64_t* mmax, uint32_t* status, uint64_t* fold_acc, uint32_t* arrivals,
                                hipStream_t stream)
{
  const MaxPlan m = plan_maxima(fold_acc, arrivals, n_tensors, n_tiles, grid, vmax, mmax, nullptr);
  if ((vmax || mmax) && !m.fold.arrivals)
    hipLaunchKernelGGL(fill2_u64_kernel, dim3((n_tensors + kBlock - 1) / kBlock), dim3(kBlock), 0, stream, vmax, mmax, n_tensors);
  if (n_tiles) {
    if (grad_is_f32)
      hipLaunchKernelGGL(momentum_step_kernel<kGradF32>, dim3(grid), dim3(kBlock), 0, stream, tensors, tiles, n_tiles,
                         fl_in, fl_out, fl_m_in, fl_m_out, fl_g, lr, mu, wd, m.acc[0], m.acc[1], status, m.fold);
    else
      hipLaunchKernelGGL(momentum_step_kernel<kGradI16>, dim3(grid), dim3(kBlock), 0, stream, tensors, tiles, n_tiles,
                         fl_in, fl_out, fl_m_in, fl_m_out, fl_g, lr, mu, wd, m.acc[0], m.acc[1], status, m.fold);
  }
  return hipGetLastError();
}

}  // namespace lpk

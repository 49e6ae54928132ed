// Fused lazy-update kernel (Algorithm 1 of the paper, Section 2): one launch
// walks every tile of every tensor of a list.
//
// Work distribution: a persistent grid of wavefronts; wave w takes tiles
// w, w + W, w + 2W, ... of the tile table, so at any moment the grid streams
// one contiguous window of the parameter set.  A tile is 4096 elements of one
// tensor; a lane handles 16 consecutive elements per pass (one dwordx4 of int8
// theta, one of comp, two of int16 grad), several passes in flight together.
//
// Stores: a 16-byte group of theta or comp that the step left unchanged is not
// written back (see "Lazy stores" below); a second kernel instance, for lists
// with LPK_OPT_STORE_ALL, writes everything.  The host launches one workgroup
// of four waves per CU for that dense read-modify-write stream (with its 2:1
// read/write byte mix HBM delivers most when few, large bursts are in flight)
// and two per CU for the read-mostly stream of the default instance.
//
// Gradient source: the int16 gradients written by the quantization kernel, or
// (further kernel instances) the fp32 gradients themselves, quantized in
// registers exactly as the quantization kernel would -- the fused form saves
// the int16 round trip through HBM.
//
// Arithmetic: three paths with identical results, chosen per tensor.
//   * wide: exact fp64, any widths / shifts / grid move / decay /
//     no-accumulator mode inside the documented domain;
//   * fast: 32-bit, when the shifts allow it.  The step
//     RNE(-lr*g / 2^k) is ONE fp32 fused multiply-add: g and lr are exact in
//     fp32, the FMA forms their product exactly and adds 1.5*2^(23+k), whose
//     ulp is 2^k, so the single IEEE rounding of the FMA *is* the
//     round-to-nearest-even at bit k and the integer falls out of the
//     significand bits.  The decay term uses the same construction in fp64;
//   * small: int8 theta with an int8 accumulator and every intermediate below
//     2^22 -- the rounding of v onto theta's grid runs on the FMA unit too.
//
// Running maximum of |v| per tensor: per-lane max, DPP wave reduction when a
// wave moves to another tensor, LDS stage across the four waves of a block at
// the end, one atomic per (block, tensor).
#include "step_common.hpp"

namespace lpk {


struct StepParams {
  int      path;            // 0 skip, 1 element by element (wide arithmetic), 2 vector (arithmetic by `mode`)
  int      wt, wc, wg, d;
  int      has_comp;
  int      kg;              // shift of the gradient term: fl_g + 16 - F
  int      kw;              // shift of the decay term: 32 - d
  int      u, kth, kc;      // grid move: v_G = v << u; theta' = RNE(v_G >> kth); c' = RNE(r >> kc)
  int64_t  lr, lrwd;
  int      qmin_t, qmax_t, qmin_c, qmax_c;
  float    gscale, glo, ghi;            // fp32 gradient source: 2^fl_g and the rails of the gradient width
  // fast path constants
  float    nlr_f;  float magic_f;  int magic_fi;
  double   nlrwd_d; double magic_d; int magic_dlo;
  Alg1Int  in;              // last stage by add-and-shift
  // small-value variant of the fast path (every |intermediate| < 2^22, d <= 8): roundings on the FMA unit
  int      bias_i;          // -bits(1.5 * 2^(23 + kg)): takes the FMA's offset out of the step
  Alg1Small sm;             // last stage on the FMA unit
  int      mode;            // vector arithmetic: kModeFast, kModeSmall or kModeWide
};

// Constants of the wide path (fp64, any shifts), built from the shifts where that path starts so that they hold
// no registers while the 32-bit loops run: -lr * 2^-kg, -lr * wd * 2^-kw, and the last stage's powers of two and rails.
struct WideParams {
  bool     decay;
  double   ag, aw;
  Alg1Wide a;
};

enum { kModeFast = 0, kModeSmall = 1, kModeWide = 2 };

// Quantize one fp32 gradient exactly as the quantization kernel does; the result is an integer-valued float.
// `ab_max` collects the largest |bit pattern| seen (>= 0x7f800000 means a NaN or Inf went by).
__device__ __forceinline__ float quant_grad(const StepParams& p, float x, uint32_t& ab_max)
{
  const uint32_t ab = __float_as_uint(x) & 0x7fffffffu;
  ab_max = ab > ab_max ? ab : ab_max;
  float y = __builtin_rintf(x * p.gscale);
  y = __builtin_fminf(__builtin_fmaxf(y, p.glo), p.ghi);
  return ab > 0x7f800000u ? 0.0f : y;                  // NaN -> 0
}

// ---------------------------------------------------------------- wide (fp64, any shifts of the domain)
//
// Every quantity of the definition is an integer below 2^53 times a power of two: |lr * g| < 2^31,
// |lr * wd * theta| < 2^47, each term capped at 2^40, |v| < 2^42.  Products, sums and scalings by powers of two are
// therefore exact in binary64, and v_rndne_f64 is the round-to-nearest-even of the definition whichever way a
// shift points -- no branches, no 64-bit integer sequences.

__device__ __forceinline__ WideParams make_wide(const StepParams& p)
{
  WideParams w;
  w.decay = p.lrwd != 0;
  w.ag = -(double)p.lr * pow2d(-p.kg);
  w.aw = -(double)p.lrwd * pow2d(-p.kw);
  w.a = make_alg1_wide(p.d, p.u, p.kth, p.kc, p.qmin_t, p.qmax_t, p.qmin_c, p.qmax_c);
  return w;
}

// DECAY is a template parameter here too: a branch per element, even a uniform one, would keep the compiler from
// interleaving the elements of a group.
template <bool DECAY>
__device__ __forceinline__ void update_wide(const WideParams& w, int th, int c, double g, int& th_new, int& c_new, double& vabs_max)
{
  const double cap = 1099511627776.0;                       // 2^40
  double s = clampd(__builtin_rint(g * w.ag), -cap, cap);
  if (DECAY) s += clampd(__builtin_rint((double)th * w.aw), -cap, cap);
  alg1_wide(w.a, th, c, s, th_new, c_new, vabs_max);
}

// Element-at-a-time tile: any alignment, any widths.  Lane l takes elements l, l+64, ...
template <int GS>
__device__ __forceinline__ uint64_t tile_generic(const StepParams& p, const TensorDev& T, uint64_t off, uint32_t cnt, int lane,
                                                 uint32_t& ab_max)
{
  double vw = 0.0;
  const WideParams w = make_wide(p);
  for (uint32_t j = lane; j < cnt; j += kWave) {
    uint64_t i = off + j;
    int th = load_elem(T.theta, i, p.wt);
    int c  = p.has_comp ? load_elem(T.comp, i, p.wc) : 0;
    int g  = GS == kGradF32 ? (int)quant_grad(p, ((const float*)T.src)[i], ab_max) : load_elem(T.grad, i, p.wg);
    int tn, cn;
    if (w.decay) update_wide<true>(w, th, c, (double)g, tn, cn, vw); else update_wide<false>(w, th, c, (double)g, tn, cn, vw);
    store_elem(T.theta, i, p.wt, tn);
    if (p.has_comp) store_elem(T.comp, i, p.wc, cn);
  }
  return (uint64_t)vw;                                   // an integer below 2^42
}

// ---------------------------------------------------------------- fast (int32 + FMA rounding)

struct Track { VTrack vt; uint32_t ab; double vw; int dense_t, dense_c; };     // dense_*: groups of this tile whose theta / comp stores went out dense

template <bool DECAY>
__device__ __forceinline__ void update_fast(const StepParams& p, int th, int c, float gf, int& tn, int& cn, Track& tr)
{
  int s = __float_as_int(__builtin_fmaf(gf, p.nlr_f, p.magic_f)) - p.magic_fi;
  if (DECAY) {
    double r = __builtin_fma((double)th, p.nlrwd_d, p.magic_d);
    s += __double2loint(r) - p.magic_dlo;
  }
  const int v = (int)((unsigned)th << p.d) + c + s;
  track_v(tr.vt, v);
  alg1_int(p.in, v, tn, cn);                                // d >= 1, no overflow by path choice
}

// The same update when every intermediate is below 2^22 in magnitude and d <= 8 (int8 theta with an int8
// accumulator), or below 2^23 under an int16 accumulator (BIGD): both roundings run on the FMA unit.  The step is
// the bit pattern of the same FMA as in update_fast minus the bit pattern of its offset (folded into one constant
// added with comp); the last stage is alg1_small.
template <bool DECAY, bool BIGD>
__device__ __forceinline__ void update_small(const StepParams& p, int th, int c, float gf, int& tn, int& cn, Track& tr)
{
  int s = __float_as_int(__builtin_fmaf(gf, p.nlr_f, p.magic_f));
  if (DECAY) {
    double r = __builtin_fma((double)th, p.nlrwd_d, p.magic_d);
    s += __double2loint(r) - p.magic_dlo;
  }
  const int v = (int)((unsigned)th << p.d) + (c + p.bias_i) + s;
  track_v(tr.vt, v);
  alg1_small<BIGD>(p.sm, v, tn, cn);
}

// 16 consecutive elements of one lane.  WT / WC = widths of theta and comp; GS = gradient source.
template <int WT, int WC, int GS> struct Group {
  v4i th[WT / 8], c[WC / 8], g[GS == kGradF32 ? 4 : (GS == kGradI8 ? 1 : 2)];
};

template <int WT, int WC, int GS>
__device__ __forceinline__ void load_group(Group<WT, WC, GS>& G, const TensorDev& T, uint64_t e)
{
  load16<WT>(G.th, T.theta, e);
  load16<WC>(G.c, T.comp, e);
  if (GS == kGradF32) {
#pragma unroll
    for (int j = 0; j < (GS == kGradF32 ? 4 : 2); ++j) G.g[j] = ld_stream((const v4i*)((const float*)T.src + e + 4 * j));
  } else if (GS == kGradI8) {
    G.g[0] = ld_stream((const v4i*)((const int8_t*)T.grad + e));
  } else {
    G.g[0] = ld_stream((const v4i*)((const int16_t*)T.grad + e));
    G.g[GS == kGradI16 ? 1 : 0] = ld_stream((const v4i*)((const int16_t*)T.grad + e + 8));
  }
}

// The packed results of one group, kept in registers until they are stored.
template <int WT, int WC> struct GroupOut { v4i th[WT / 8], c[WC / 8]; };

template <int W> __device__ __forceinline__ void pack16(v4i (&dst)[W / 8], const int (&val)[16])
{
  if (W == 8) {
#pragma unroll
    for (int w = 0; w < 4; ++w) dst[0][w] = pack4x8(val[4 * w], val[4 * w + 1], val[4 * w + 2], val[4 * w + 3]);
  } else {
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
      for (int w = 0; w < 4; ++w) dst[(W / 8 - 1) * q][w] = pack2x16(val[8 * q + 2 * w], val[8 * q + 2 * w + 1]);
  }
}
template <int W> __device__ __forceinline__ void store16v(void* base, uint64_t e, const v4i (&src)[W / 8])
{
  if (W == 8) st_stream((v4i*)((int8_t*)base + e), src[0]);
  else { st_stream((v4i*)((int16_t*)base + e), src[0]); st_stream((v4i*)((int16_t*)base + e + 8), src[W / 8 - 1]); }
}

template <int WT, int WC, int GS, bool DECAY, int MODE>
__device__ __forceinline__ void compute_group(const StepParams& p, const WideParams& w, const Group<WT, WC, GS>& G, GroupOut<WT, WC>& O, Track& tr)
{
  int tn[16], cn[16];
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    float gf;
    if (GS == kGradF32) gf = quant_grad(p, __int_as_float(G.g[(k >> 2) & (GS == kGradF32 ? 3 : 1)][k & 3]), tr.ab);
    else if (GS == kGradI8) gf = (float)sx8(G.g[0][k >> 2], k & 3);
    else                gf = (float)sx16(G.g[(k >> 3) & (GS == kGradI16 ? 1 : 0)][(k >> 1) & 3], k & 1);
    if (MODE == kModeSmall)     update_small<DECAY, (WC == 16)>(p, elem16<WT>(G.th, k), elem16<WC>(G.c, k), gf, tn[k], cn[k], tr);
    else if (MODE == kModeWide) update_wide<DECAY>(w, elem16<WT>(G.th, k), elem16<WC>(G.c, k), (double)gf, tn[k], cn[k], tr.vw);
    else                        update_fast<DECAY>(p, elem16<WT>(G.th, k), elem16<WC>(G.c, k), gf, tn[k], cn[k], tr);
  }
  pack16<WT>(O.th, tn);
  pack16<WC>(O.c, cn);
}

template <int WT, int WC>
__device__ __forceinline__ void store_group(const GroupOut<WT, WC>& O, const TensorDev& T, uint64_t e)
{
  store16v<WT>(T.theta, e, O.th);
  store16v<WC>(T.comp, e, O.c);
}

// Lazy stores.  In the lazy update most parameters do not move in a step (that is its premise: a step is usually
// far below the parameter's grid, and often below the accumulator's), so most 16-byte groups a lane computes equal
// the ones it loaded and need not be written back (lazy_store).  The tile functions exist in three forms (LAZY):
// kLazyBoth tests theta and comp, kLazyTheta tests theta only (a step around one accumulator LSB changes most of
// comp and hardly any theta), kLazyNone tests nothing.  A wave whose tile turned out mostly dense in comp, or in
// theta too, runs its next kDenseTiles tiles through the form that no longer tests that array, then probes again:
// this keeps the cost of the tests out of workloads where everything changes.  The kernel instance for lists with
// LPK_OPT_STORE_ALL only holds kLazyNone.
constexpr int kDenseTiles = 16;
enum { kLazyNone = 0, kLazyTheta = 1, kLazyBoth = 2 };
struct LazyRun { int tiles, form; };                        // a wave's state across tiles: `tiles` more tiles in `form`

template <int W> __device__ __forceinline__ bool store16_lazy(void* base, uint64_t e, const v4i (&o)[W / 8], const v4i (&in)[W / 8])
{
  int x = 0;
#pragma unroll
  for (int q = 0; q < W / 8; ++q)
#pragma unroll
    for (int k = 0; k < 4; ++k) x |= o[q][k] ^ in[q][k];
  return lazy_store<16>(x != 0, [&] { store16v<W>(base, e, o); });
}

template <int WT, int WC, int LAZY>
__device__ __forceinline__ void store_group_lazy(const GroupOut<WT, WC>& O, const v4i (&th_in)[WT / 8], const v4i (&c_in)[WC / 8], const TensorDev& T, uint64_t e, Track& tr)
{
  if (LAZY == kLazyNone) store16v<WT>(T.theta, e, O.th); else tr.dense_t += store16_lazy<WT>(T.theta, e, O.th, th_in) ? 1 : 0;
  if (LAZY != kLazyBoth) store16v<WC>(T.comp, e, O.c);   else tr.dense_c += store16_lazy<WC>(T.comp, e, O.c, c_in) ? 1 : 0;
}

template <int WT, int WC, int GS, bool DECAY, int MODE, int LAZY>
__device__ __forceinline__ void compute_store_group(const StepParams& p, const WideParams& w, const Group<WT, WC, GS>& G, const TensorDev& T, uint64_t e, Track& tr)
{
  GroupOut<WT, WC> O;
  compute_group<WT, WC, GS, DECAY, MODE>(p, w, G, O, tr);
  store_group_lazy<WT, WC, LAZY>(O, G.th, G.c, T, e, tr);
}

__device__ __forceinline__ uint64_t track_max(const Track& tr)
{
  const uint64_t m32 = vtrack_max(tr.vt), m64 = (uint64_t)tr.vw;
  return m32 > m64 ? m32 : m64;
}

// Vector tile: full 16-element groups with the fast arithmetic, the ragged end element by element.
template <int WT, int WC, int GS, bool DECAY, int MODE, int LAZY>
__device__ __forceinline__ uint64_t tile_fast(const StepParams& p, const TensorDev& T, uint64_t off, uint32_t cnt, int lane, uint32_t& ab_max, LazyRun& lz)
{
  Track tr{{0, 0}, ab_max, 0.0, 0, 0};
  const WideParams w = MODE == kModeWide ? make_wide(p) : WideParams{};
  constexpr int kRegs = (WT + WC) / 2 + (GS == kGradF32 ? 16 : (GS == kGradI8 ? 4 : 8));     // VGPRs of one group
  constexpr int kP = kRegs <= 16 ? (LAZY == kLazyNone ? LPK_I16_GROUPS : LPK_I16_GROUPS_LAZY) : LPK_KP_WIDE;   // groups in flight per lane
  const uint32_t ngroups = cnt / kGroup;
  uint32_t gi = lane;
  for (; gi + (kP - 1) * kWave < ngroups; gi += kP * kWave) {             // kP groups in flight: all loads, then compute and store
    Group<WT, WC, GS> G[kP];
#pragma unroll
    for (int ps = 0; ps < kP; ++ps) load_group(G[ps], T, off + (uint64_t)(gi + ps * kWave) * kGroup);
#pragma unroll
    for (int ps = 0; ps < kP; ++ps) compute_store_group<WT, WC, GS, DECAY, MODE, LAZY>(p, w, G[ps], T, off + (uint64_t)(gi + ps * kWave) * kGroup, tr);
  }
  for (; gi < ngroups; gi += kWave) {
    Group<WT, WC, GS> G;
    const uint64_t e = off + (uint64_t)gi * kGroup;
    load_group(G, T, e);
    compute_store_group<WT, WC, GS, DECAY, MODE, LAZY>(p, w, G, T, e, tr);
  }
  ab_max = tr.ab;
  if (LAZY != kLazyNone) {                                 // most of this tile's groups dense in theta / in comp?
    const bool mt = 2 * (uint32_t)wave_uniform(tr.dense_t) * kWave > ngroups, mc = 2 * (uint32_t)wave_uniform(tr.dense_c) * kWave > ngroups;
    if (mt)      { lz.tiles = kDenseTiles; lz.form = kLazyNone; }
    else if (mc) { lz.tiles = kDenseTiles; lz.form = kLazyTheta; }
  }
  uint64_t vm = track_max(tr);
  const uint32_t tail = cnt - ngroups * kGroup;           // < 16 elements
  if (tail) {
    uint64_t t2 = tile_generic<GS>(p, T, off + (uint64_t)ngroups * kGroup, tail, lane, ab_max);
    vm = t2 > vm ? t2 : vm;
  }
  return vm;
}

// ---------------------------------------------------------------- E consecutive elements per lane
//
// How many consecutive elements one lane owns decides which of its loads are fully coalesced.  With fp32
// gradients, 16 per lane would mean 64 contiguous bytes of gradients per lane (four loads whose lanes sit 64
// bytes apart), which the memory pipeline handles far worse than HBM itself; fewer elements per lane trade
// wider gradient accesses for narrower theta/comp accesses.  This path is generic in E (4, 8 or 16).

template <int E, int WT, int WC, int GS> struct GroupE {
  static constexpr int kG = GS == kGradF32 ? E / 4 : (GS == kGradI8 ? 1 : (E >= 8 ? E / 8 : 1));      // gradient accesses
  static constexpr int kGN = GS == kGradF32 ? 4 : (GS == kGradI8 ? E / 4 : (E >= 8 ? 4 : 2));         // dwords per gradient access
  DW<E * WT / 32> th;
  DW<E * WC / 32> c;
  DW<kGN> g[kG];
};

template <int E, int WT, int WC, int GS>
__device__ __forceinline__ void load_group_e(GroupE<E, WT, WC, GS>& G, const TensorDev& T, uint64_t e)
{
  using GT = GroupE<E, WT, WC, GS>;
  G.th = ld_dw<E * WT / 32>((const int8_t*)T.theta + e * (WT / 8));
  G.c  = ld_dw<E * WC / 32>((const int8_t*)T.comp + e * (WC / 8));
#pragma unroll
  for (int j = 0; j < GT::kG; ++j) {
    if constexpr (GS == kGradF32)     G.g[j] = ld_dw<4>((const float*)T.src + e + 4 * j);
    else if constexpr (GS == kGradI8) G.g[j] = ld_dw<GT::kGN>((const int8_t*)T.grad + e);
    else                              G.g[j] = ld_dw<GT::kGN>((const int16_t*)T.grad + e + 8 * j);
  }
}

template <int E, int WT, int WC> struct GroupOutE { DW<E * WT / 32> th; DW<E * WC / 32> c; };

template <int E, int WT, int WC, int GS, bool DECAY, int MODE>
__device__ __forceinline__ void compute_group_e(const StepParams& p, const WideParams& w, const GroupE<E, WT, WC, GS>& G, GroupOutE<E, WT, WC>& O, Track& tr)
{
  int tn[E], cn[E];
#pragma unroll
  for (int k = 0; k < E; ++k) {
    float gf;
    if constexpr (GS == kGradF32) gf = quant_grad(p, __int_as_float(G.g[k >> 2].d[k & 3]), tr.ab);
    else if constexpr (GS == kGradI8) gf = (float)sx8(G.g[0].d[k >> 2], k & 3);
    else                          gf = (float)sx16(G.g[k >> 3].d[(k >> 1) & 3], k & 1);
    if constexpr (MODE == kModeSmall)     update_small<DECAY, (WC == 16)>(p, elem_dw<WT>(G.th, k), elem_dw<WC>(G.c, k), gf, tn[k], cn[k], tr);
    else if constexpr (MODE == kModeWide) update_wide<DECAY>(w, elem_dw<WT>(G.th, k), elem_dw<WC>(G.c, k), (double)gf, tn[k], cn[k], tr.vw);
    else                                  update_fast<DECAY>(p, elem_dw<WT>(G.th, k), elem_dw<WC>(G.c, k), gf, tn[k], cn[k], tr);
  }
  O.th = pack_dw<WT, E>(tn);
  O.c  = pack_dw<WC, E>(cn);
}

template <int E, int WT, int WC, int GS, int LAZY>
__device__ __forceinline__ void store_group_e(const GroupOutE<E, WT, WC>& O, const GroupE<E, WT, WC, GS>& G, const TensorDev& T, uint64_t e, Track& tr)
{
  if constexpr (LAZY == kLazyNone) st_dw((int8_t*)T.theta + e * (WT / 8), O.th);
  else tr.dense_t += st_dw_lazy((int8_t*)T.theta + e * (WT / 8), O.th, G.th) ? 1 : 0;
  if constexpr (LAZY != kLazyBoth) st_dw((int8_t*)T.comp + e * (WC / 8), O.c);
  else tr.dense_c += st_dw_lazy((int8_t*)T.comp + e * (WC / 8), O.c, G.c) ? 1 : 0;
}

template <int E, int WT, int WC, int GS, bool DECAY, int MODE, int LAZY>
__device__ __forceinline__ void compute_store_group_e(const StepParams& p, const WideParams& w, const GroupE<E, WT, WC, GS>& G, const TensorDev& T, uint64_t e, Track& tr)
{
  GroupOutE<E, WT, WC> O;
  compute_group_e<E, WT, WC, GS, DECAY, MODE>(p, w, G, O, tr);
  store_group_e<E, WT, WC, GS, LAZY>(O, G, T, e, tr);
}

template <int E, int KP, int WT, int WC, int GS, bool DECAY, int MODE, int LAZY>
__device__ __forceinline__ uint64_t tile_fast_e(const StepParams& p, const TensorDev& T, uint64_t off, uint32_t cnt, int lane, uint32_t& ab_max, LazyRun& lz)
{
  Track tr{{0, 0}, ab_max, 0.0, 0, 0};
  const WideParams w = MODE == kModeWide ? make_wide(p) : WideParams{};
  const uint32_t ngroups = cnt / E;
  uint32_t gi = lane;
  for (; gi + (KP - 1) * kWave < ngroups; gi += KP * kWave) {             // KP groups in flight: all loads, then compute and store
    GroupE<E, WT, WC, GS> G[KP];
#pragma unroll
    for (int ps = 0; ps < KP; ++ps) load_group_e(G[ps], T, off + (uint64_t)(gi + ps * kWave) * E);
#pragma unroll
    for (int ps = 0; ps < KP; ++ps) compute_store_group_e<E, WT, WC, GS, DECAY, MODE, LAZY>(p, w, G[ps], T, off + (uint64_t)(gi + ps * kWave) * E, tr);
  }
  for (; gi < ngroups; gi += kWave) {
    GroupE<E, WT, WC, GS> G;
    const uint64_t e = off + (uint64_t)gi * E;
    load_group_e(G, T, e);
    compute_store_group_e<E, WT, WC, GS, DECAY, MODE, LAZY>(p, w, G, T, e, tr);
  }
  ab_max = tr.ab;
  if (LAZY != kLazyNone) {                                 // most of this tile's groups dense in theta / in comp?
    const bool mt = 2 * (uint32_t)wave_uniform(tr.dense_t) * kWave > ngroups, mc = 2 * (uint32_t)wave_uniform(tr.dense_c) * kWave > ngroups;
    if (mt)      { lz.tiles = kDenseTiles; lz.form = kLazyNone; }
    else if (mc) { lz.tiles = kDenseTiles; lz.form = kLazyTheta; }
  }
  uint64_t vm = track_max(tr);
  const uint32_t tail = cnt - ngroups * E;                // < E elements
  if (tail) {
    uint64_t t2 = tile_generic<GS>(p, T, off + (uint64_t)ngroups * E, tail, lane, ab_max);
    vm = t2 > vm ? t2 : vm;
  }
  return vm;
}

// ---------------------------------------------------------------- per-tensor set-up (wave-uniform)

template <int GS, bool WITH_I8>
__device__ __forceinline__ void setup_tensor(StepParams& p, const TensorDev& T, int fl_in, int fl_out, int fl_g,
                                             uint32_t lr, uint32_t wd, uint32_t& status_bits)
{
  p.wt = T.wt; p.wc = T.wc; p.wg = T.wg; p.has_comp = T.comp != nullptr;
  p.d = p.has_comp ? T.d : 0;
  const int delta = fl_out - fl_in;
  if (fl_in < kFlMin || fl_in > kFlMax || fl_out < kFlMin || fl_out > kFlMax || fl_g < kFlMin || fl_g > kFlMax ||
      p.d > kDMax || delta > kDeltaMax || delta < -kDeltaMax) {
    p.path = skipped_path<GS>(fl_g); status_bits |= kStatusDomain; return;
  }
  const int F = fl_in + p.d;
  p.kg = fl_g + 16 - F;
  p.kw = 32 - p.d;
  p.u = delta > 0 ? delta : 0;
  p.kth = p.d + p.u - delta;
  p.kc = p.kth - p.d;
  p.lr = lr; p.lrwd = (int64_t)lr * (int64_t)wd;
  p.qmax_t = (1 << (p.wt - 1)) - 1; p.qmin_t = -(1 << (p.wt - 1));
  const int wc = p.has_comp ? p.wc : 8;
  p.qmax_c = (1 << (wc - 1)) - 1;   p.qmin_c = -(1 << (wc - 1));
  p.gscale = __uint_as_float((uint32_t)(127 + fl_g) << 23);
  p.glo = -(float)(1 << (p.wg - 1)); p.ghi = (float)((1 << (p.wg - 1)) - 1);
  p.path = 1; p.mode = kModeWide;

  // Vector path: theta, comp and 16-bit gradients on 16-byte aligned buffers, comp as wide as theta (or int8 theta
  // with an int16 accumulator).  Its arithmetic is the wide one unless the shifts allow 32 bits:
  // no grid move, 1 <= d, a step shift k with |lr * g| <= lr * 2^15 < 2^(22+k) (so the fp32 FMA rounding trick
  // is exact and |s| < 2^22), and every intermediate provably inside int32.
  const bool widths_ok = (p.wt == p.wc) || (p.wt == 8 && p.wc == 16);
  const bool vec = T.vec_step && (GS == kGradI16 || (((uintptr_t)T.src) & 15u) == 0);
  // gradients: 16 bits wide, or (int8 array next to an 8-bit theta) 8 bits wide
  // (from the fp32 source the width only sets the rails of the quantization)
  const bool grads_ok = p.wg == 16 || (GS == kGradF32 && p.wg == 8) || (WITH_I8 && GS == kGradI16 && p.wg == 8 && p.wt == 8);
  if (!p.has_comp || !vec || !widths_ok || !grads_ok) return;
  p.path = 2;
  if (delta != 0 || p.d < 1 || p.kg < 1) return;
  if (p.kg < 9 && ((int64_t)lr << 15) >= (1ll << (22 + p.kg))) return;
  int64_t bound = (1ll << (p.wt - 1 + p.d)) + (1ll << (p.wc - 1));             // |theta * 2^d| + |c|
  bound += p.kg < 40 ? (((int64_t)lr << 15) >> p.kg) + 1 : 0;                   // |s_g|
  int64_t sw = 0;
  if (p.lrwd) sw = ((p.lrwd << (p.wt - 1)) >> p.kw) + 1;                        // |s_w|
  bound += sw;
  bound += 1ll << (p.d - 1);                                                    // the rounding addend
  if (bound >= (1ll << 31)) return;
  p.mode = kModeFast;
  const int kg = p.kg > 40 ? 40 : p.kg;                                         // k >= 32 already gives s = 0
  p.magic_fi = ((127 + 23 + kg) << 23) | 0x400000;                              // 1.5 * 2^(23 + k)
  p.magic_f  = __int_as_float(p.magic_fi);
  p.nlr_f    = -(float)lr;
  const long long md = ((long long)(1023 + 52 + p.kw) << 52) | (1ll << 51);     // 1.5 * 2^(52 + kw)
  p.magic_d   = __longlong_as_double(md);
  p.magic_dlo = (int)(md & 0xffffffffll);
  p.nlrwd_d   = -(double)p.lrwd;
  p.in = Alg1Int{p.d, (1 << (p.d - 1)) - 1, p.qmin_t, p.qmax_t, p.qmin_c, p.qmax_c};
  // small-value variant, int8 theta: |v| plus the rounding addend below 2^22 and (2^22 + theta') * 2^d inside int32
  // (int8 accumulator, d <= 8), or below 2^23 with the residual formed unshifted (int16 accumulator, d <= 22);
  // either way v is exact in fp32 and the quotient sits inside the 2^22 window of the 1.5 * 2^23 offset
  if (p.wt == 8 && p.wc == 8 && p.d <= 8 && bound < (1ll << 22)) p.mode = kModeSmall;
  if (p.wt == 8 && p.wc == 16 && p.d <= 22 && bound < (1ll << 23)) p.mode = kModeSmall;
  p.bias_i  = -p.magic_fi;
  p.sm = make_alg1_small(p.d, p.qmin_t, p.qmax_t, p.qmin_c, p.qmax_c);
}

// ---------------------------------------------------------------- the kernel

template <int WT, int WC, int GS, int MODE, int LAZY>
__device__ __forceinline__ uint64_t tile_fast_decay(const StepParams& p, const TensorDev& T, uint64_t off, uint32_t cnt, int lane, uint32_t& ab, LazyRun& lz)
{
  const bool decay = p.lrwd != 0;
  // the wide arithmetic: 8 elements per lane, one group in flight -- its fp64 temporaries would otherwise set the
  // register count of the whole kernel, and the 32-bit loops lose speed above about 160 VGPRs
  if constexpr (MODE == kModeWide)
    return decay ? tile_fast_e<8, 1, WT, WC, GS, true, MODE, kLazyNone>(p, T, off, cnt, lane, ab, lz)
                 : tile_fast_e<8, 1, WT, WC, GS, false, MODE, kLazyNone>(p, T, off, cnt, lane, ab, lz);
  // fp32 gradients: 8 elements per lane (two dwordx4 of gradients), four groups in flight when everything is stored,
  // two when only theta's stores are tested (comp written densely); 4 per lane (one fully coalesced dwordx4 of
  // gradients, one dword of theta and of comp) with eight groups in flight when both arrays' stores are tested --
  // 8 % faster on that read-mostly stream, 2-4 % slower on the other two
  if constexpr (GS == kGradF32 && LAZY == kLazyBoth)
    return decay ? tile_fast_e<LPK_F32_E_BOTH, LPK_F32_GROUPS_BOTH, WT, WC, GS, true, MODE, LAZY>(p, T, off, cnt, lane, ab, lz)
                 : tile_fast_e<LPK_F32_E_BOTH, LPK_F32_GROUPS_BOTH, WT, WC, GS, false, MODE, LAZY>(p, T, off, cnt, lane, ab, lz);
  if (GS == kGradF32)
    return decay ? tile_fast_e<LPK_F32_E, (LAZY == kLazyNone ? LPK_F32_GROUPS : LPK_F32_GROUPS_LAZY), WT, WC, GS, true, MODE, LAZY>(p, T, off, cnt, lane, ab, lz)
                 : tile_fast_e<LPK_F32_E, (LAZY == kLazyNone ? LPK_F32_GROUPS : LPK_F32_GROUPS_LAZY), WT, WC, GS, false, MODE, LAZY>(p, T, off, cnt, lane, ab, lz);
#if LPK_I16_E != 16
  return decay ? tile_fast_e<LPK_I16_E, (LAZY == kLazyNone ? LPK_I16_GROUPS : LPK_I16_GROUPS_LAZY), WT, WC, GS, true, MODE, LAZY>(p, T, off, cnt, lane, ab, lz)
               : tile_fast_e<LPK_I16_E, (LAZY == kLazyNone ? LPK_I16_GROUPS : LPK_I16_GROUPS_LAZY), WT, WC, GS, false, MODE, LAZY>(p, T, off, cnt, lane, ab, lz);
#endif
  // 8-bit theta and comp while both arrays' stores are tested (few groups change): 8 elements per lane, four groups
  // in flight -- the same bytes in flight as 16 per lane with two groups, in narrower accesses, measured 3 % faster
  // on that read-mostly stream with scattered writes (and 5 % slower once comp is written densely, which is why the
  // other forms keep 16 per lane)
  if constexpr (WC == 8 && LAZY == kLazyBoth)
    return decay ? tile_fast_e<LPK_I8_E_BOTH, LPK_I8_GROUPS_BOTH, WT, WC, GS, true, MODE, LAZY>(p, T, off, cnt, lane, ab, lz)
                 : tile_fast_e<LPK_I8_E_BOTH, LPK_I8_GROUPS_BOTH, WT, WC, GS, false, MODE, LAZY>(p, T, off, cnt, lane, ab, lz);
  // a 16-bit theta or comp: 8 elements per lane, so that every access of a wave is one contiguous run (with 16, a
  // lane's 16-bit data spans two stores 32 bytes apart and HBM sees partial-line writes)
  if constexpr (WC == 16)
    return decay ? tile_fast_e<8, (LAZY == kLazyNone ? LPK_W16_GROUPS : LPK_W16_GROUPS_LAZY), WT, WC, GS, true, MODE, LAZY>(p, T, off, cnt, lane, ab, lz)
                 : tile_fast_e<8, (LAZY == kLazyNone ? LPK_W16_GROUPS : LPK_W16_GROUPS_LAZY), WT, WC, GS, false, MODE, LAZY>(p, T, off, cnt, lane, ab, lz);
  return decay ? tile_fast<WT, WC, GS, true, MODE, LAZY>(p, T, off, cnt, lane, ab, lz)
               : tile_fast<WT, WC, GS, false, MODE, LAZY>(p, T, off, cnt, lane, ab, lz);
}

template <int WT, int WC, int GS, int LAZY>
__device__ __forceinline__ uint64_t tile_vector_mode(const StepParams& p, const TensorDev& T, uint64_t off, uint32_t cnt, int lane, uint32_t& ab, LazyRun& lz)
{
  if (p.mode == kModeWide) return tile_fast_decay<WT, WC, GS, kModeWide, kLazyNone>(p, T, off, cnt, lane, ab, lz);
  if (WT == 8 && p.mode == kModeSmall) return tile_fast_decay<WT, WC, GS, kModeSmall, LAZY>(p, T, off, cnt, lane, ab, lz);
  return tile_fast_decay<WT, WC, GS, kModeFast, LAZY>(p, T, off, cnt, lane, ab, lz);
}

template <int WT, int WC, int GS, bool STORE_ALL>
__device__ __forceinline__ uint64_t tile_vector(const StepParams& p, const TensorDev& T, uint64_t off, uint32_t cnt, int lane, uint32_t& ab, LazyRun& lz)
{
  if constexpr (STORE_ALL) return tile_vector_mode<WT, WC, GS, kLazyNone>(p, T, off, cnt, lane, ab, lz);
  if (lz.tiles > 0) {                                      // inside a dense run
    --lz.tiles;
    if (lz.form == kLazyNone) return tile_vector_mode<WT, WC, GS, kLazyNone>(p, T, off, cnt, lane, ab, lz);
    return tile_vector_mode<WT, WC, GS, kLazyTheta>(p, T, off, cnt, lane, ab, lz);
  }
  return tile_vector_mode<WT, WC, GS, kLazyBoth>(p, T, off, cnt, lane, ab, lz);
}

// STORE_ALL: the instance for lists with LPK_OPT_STORE_ALL, which holds none of the store tests.
// WITH_I8: the instance for lists that hold int8 gradient arrays (their vector path stays out of the others' code).
template <int GS, bool STORE_ALL, bool WITH_I8>
__global__ void __launch_bounds__(kBlock)
kahan_step_kernel(const TensorDev* __restrict__ tensors, const Tile* __restrict__ tiles, uint32_t n_tiles,
                  const int32_t* __restrict__ fl_in, const int32_t* __restrict__ fl_out, const int32_t* __restrict__ fl_g,
                  uint32_t lr, uint32_t wd, uint64_t* vmax, uint32_t* status, MaxFold fold)
{
  __shared__ int      s_tensor[kWavesPerBlock];
  __shared__ uint64_t s_max[kWavesPerBlock];

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = wave_uniform(threadIdx.x >> 6);

  uint64_t lane_max = 0;
  uint32_t status_bits = 0, ab_max = 0;
  StepParams p; p.path = 0;
  TensorDev T;
  LazyRun lz{0, kLazyNone};

  const int cur = walk_tiles(tiles, n_tiles,
    [&](int t) LPK_INLINE_LAMBDA { if (vmax) flush_wave(vmax, t, lane_max, lane); },
    [&](int t) LPK_INLINE_LAMBDA {
      lane_max = 0;
      T = tensors[t];
      setup_tensor<GS, WITH_I8>(p, T, fl_in[t], fl_out[t], fl_g[t], lr, wd, status_bits);
    },
    [&](uint64_t off, uint32_t cnt) LPK_INLINE_LAMBDA {
      uint64_t vm = 0;
      if (p.path == 2) {
        if (WITH_I8 && p.wt == 8 && GS == kGradI16 && p.wg == 8) {       // int8 gradient array (8-bit training mode)
          constexpr int G8 = GS == kGradI16 ? kGradI8 : GS;
          if (p.wc == 8) vm = tile_vector<8, 8, G8, STORE_ALL>(p, T, off, cnt, lane, ab_max, lz);
          else           vm = tile_vector<8, 16, G8, STORE_ALL>(p, T, off, cnt, lane, ab_max, lz);
        }
        else if (p.wt == 8 && p.wc == 8) vm = tile_vector<8, 8, GS, STORE_ALL>(p, T, off, cnt, lane, ab_max, lz);
        else if (p.wt == 16)             vm = tile_vector<16, 16, GS, STORE_ALL>(p, T, off, cnt, lane, ab_max, lz);
        else                             vm = tile_vector<8, 16, GS, STORE_ALL>(p, T, off, cnt, lane, ab_max, lz);
      } else if (p.path == 1) {
        vm = tile_generic<GS>(p, T, off, cnt, lane, ab_max);
      } else if (GS == kGradF32 && p.path == kPathSkipButScan) {
        scan_nonfinite(T.src, off, cnt, lane, ab_max);
      }
      lane_max = vm > lane_max ? vm : lane_max;
    });

  if (GS == kGradF32 && __ballot(ab_max >= 0x7f800000u)) status_bits |= kStatusNonFinite;
  raise_status(status, status_bits, lane);

  // LDS stage: the four waves of a block usually end on the same tensor.
  if (vmax) flush_block(vmax, cur, lane_max, lane, wave, s_tensor, s_max);
  if (fold.arrivals) { uint64_t* const acc[1] = {vmax}; fold_maxima<1>(fold, acc, &s_tensor[0]); }
}

__global__ void __launch_bounds__(kBlock) fill_u64_kernel(uint64_t* p, uint32_t n, uint64_t v)
{
  uint32_t i = blockIdx.x * kBlock + threadIdx.x;
  if (i < n) p[i] = v;
}

// `fold_acc`, `arrivals`: the list's accumulators for per-tensor maxima and its workgroup counter (see plan_maxima),
// or nullptr for a launch that has none.
hipError_t launch_kahan_step(const TensorDev* tensors, const Tile* tiles, uint32_t n_tiles, uint32_t n_tensors, uint32_t grid,
                             int grad_is_f32, const int32_t* fl_in, const int32_t* fl_out, const int32_t* fl_g,
                             uint32_t lr, uint32_t wd, uint32_t store_all, uint32_t with_i8, uint64_t* vmax, uint32_t* status,
                             uint64_t* fold_acc, uint32_t* arrivals, hipStream_t stream)
{
  const MaxPlan m = plan_maxima(fold_acc, arrivals, n_tensors, n_tiles, grid, vmax, nullptr, nullptr);
  if (vmax && !m.fold.arrivals)
    hipLaunchKernelGGL(fill_u64_kernel, dim3((n_tensors + kBlock - 1) / kBlock), dim3(kBlock), 0, stream, vmax, n_tensors, 0ull);
  if (n_tiles) {
    auto go = [&](auto kernel) {
      hipLaunchKernelGGL(kernel, dim3(grid), dim3(kBlock), 0, stream, tensors, tiles, n_tiles, fl_in, fl_out, fl_g, lr, wd, m.acc[0], status, m.fold);
    };
    if (grad_is_f32)  { if (store_all) go(kahan_step_kernel<kGradF32, true, false>); else go(kahan_step_kernel<kGradF32, false, false>); }
    else if (with_i8) { if (store_all) go(kahan_step_kernel<kGradI16, true, true>);  else go(kahan_step_kernel<kGradI16, false, true>); }
    else              { if (store_all) go(kahan_step_kernel<kGradI16, true, false>); else go(kahan_step_kernel<kGradI16, false, false>); }
  }
  return hipGetLastError();
}

}  // namespace lpk

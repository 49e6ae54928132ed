"""Pins of the CPU oracle to what the paper and arithmetic fix (CPU only).

Each test names the passage it checks.  None of them re-types the oracle's
integer formula: they use hand-derived values, closed forms, conservation
laws, Python's own round-half-even on Fractions, and torch.round.
"""
import os
from fractions import Fraction as Fr

import numpy as np
import pytest
import torch

from oracle import ref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def one(val, dtype):
    return np.array([val], dtype=dtype)


# ---- Section 2 / Algorithm 1: the accumulator carries sub-LSB steps -------------------------------

def load_quarter_lsb():
    rows = []
    for line in open(os.path.join(GOLDEN, "quarter_lsb_example.txt")):
        if line.strip() and not line.startswith("#"):
            rows.append(tuple(int(t) for t in line.split()))
    return rows


@pytest.mark.parametrize("sign", [+1, -1])
def test_quarter_lsb_worked_example(sign):
    """A constant step of 1/4 parameter LSB moves theta by exactly one LSB in every 4 steps."""
    theta, comp = one(0, np.int8), one(0, np.int8)
    grad = one(-sign, np.int16)
    rows = load_quarter_lsb()
    for step, t_want, c_want in rows:
        ref.kahan_sgd_step(theta, comp, grad, 7, 7, 7, 8, 32768)
        assert (int(theta[0]), int(comp[0])) == (sign * t_want, sign * c_want), step
    # keep going: theta_{4k} = k, and exactly one unit move inside every block of four steps
    prev = int(theta[0])
    for step in range(len(rows) + 1, 401):
        ref.kahan_sgd_step(theta, comp, grad, 7, 7, 7, 8, 32768)
        if step % 4 == 0:
            assert int(theta[0]) == sign * step // 4 and int(comp[0]) == 0
            assert abs(int(theta[0]) - prev) == 1
            prev = int(theta[0])


def test_quarter_lsb_without_accumulator_never_moves():
    """Eq. 1 in limited precision: a step below half an LSB vanishes every time (the failing INT8 column)."""
    theta, grad = one(0, np.int8), one(-1, np.int16)
    for _ in range(1000):
        ref.kahan_sgd_step(theta, None, grad, 0, 7, 7, 8, 32768)
    assert int(theta[0]) == 0


# ---- Section 2 / Figure 1: effective width m + n - 2 - k -------------------------------------------

@pytest.mark.parametrize("tb,cb", [(8, 8), (16, 16), (8, 16)])
def test_effective_width_closed_form(tb, cb):
    """With no overlapping bit (k = 0, d = n - 1) the pair resolves (m-1) + (n-1) magnitude bits:
    one compensation LSB per step adds up to one parameter LSB after exactly 2^(n-1) steps
    (8+16 bits -> 22, the paper's example), and half of that is below the pair's resolution."""
    d = cb - 1
    tdt, cdt = {8: np.int8, 16: np.int16}[tb], {8: np.int8, 16: np.int16}[cb]
    theta, comp, grad = one(0, tdt), one(0, cdt), one(-1, np.int16)
    fl_t = 3
    # step = lr_q * 2^-16 * 2^-fl_g = 2^-(fl_t + d)  with lr_q = 2^15  ->  fl_g = fl_t + d - 1
    fl_g = fl_t + d - 1
    n_steps = 2 ** d
    moves = []
    for i in range(1, n_steps + 1):
        ref.kahan_sgd_step(theta, comp, grad, d, fl_t, fl_t, fl_g, 32768)
        if int(theta[0]) == 1 and not moves:
            moves.append(i)
    assert int(theta[0]) == 1 and int(comp[0]) == 0
    assert moves == [n_steps // 2 + 1]          # the tie at exactly 1/2 stays on the even side
    assert (tb - 1) + (cb - 1) == tb + cb - 2 - 0
    # half a compensation LSB: lost forever
    theta[0] = 0; comp[0] = 0
    for _ in range(1000):
        ref.kahan_sgd_step(theta, comp, grad, d, fl_t, fl_t, fl_g + 1, 32768)
    assert int(theta[0]) == 0 and int(comp[0]) == 0


# ---- Kahan conservation ------------------------------------------------------------------------------

def frac_rne(x):
    return round(Fr(x))           # Python rounds Fractions half-to-even


@pytest.mark.parametrize("tb", [8, 16])
def test_conservation_invariant(tb):
    """theta*2^d + c equals the initial value plus the running sum of the quantized steps, exactly,
    as long as nothing saturates; |c| <= 2^(d-1); and theta + c follows the unquantized running sum
    to within half a compensation LSB per step."""
    rng = np.random.default_rng(3)
    dt = {8: np.int8, 16: np.int16}[tb]
    d, n, T = tb - 1, 64, 300
    fl_t, fl_g, lr_q = 6, 14, 3277
    lim = 2 ** (tb - 3)
    theta = rng.integers(-lim, lim, size=n).astype(dt)
    comp = np.zeros(n, dtype=dt)
    total_q = [int(t) * 2 ** d for t in theta]
    total_exact = [Fr(int(t) * 2 ** d) for t in theta]
    F = fl_t + d
    for step in range(T):
        g = rng.integers(-3000, 3000, size=n).astype(np.int16)
        vmax = ref.kahan_sgd_step(theta, comp, g, d, fl_t, fl_t, fl_g, lr_q)
        for i in range(n):
            step_real = -Fr(lr_q, 2 ** 16) * Fr(int(g[i]), 2 ** fl_g)       # real-valued step
            total_exact[i] += step_real * 2 ** F
            total_q[i] += frac_rne(step_real * 2 ** F)
            have = int(theta[i]) * 2 ** d + int(comp[i])
            assert have == total_q[i]
            assert abs(int(comp[i])) <= 2 ** (d - 1)
            assert abs(have - total_exact[i]) <= Fr(step + 1, 2)
        assert vmax == max(abs(v) for v in total_q)
    assert np.abs(theta.astype(np.int64)).max() < 2 ** (tb - 1) - 1     # the premise: no saturation


def test_grid_coarsening_costs_at_most_one_new_lsb():
    """When the grid gets coarser (fl_out < fl_in) the value theta + c moves by at most half a NEW
    compensation LSB beyond the step itself."""
    rng = np.random.default_rng(4)
    for _ in range(200):
        d, fl_in, delta = 7, 8, -int(rng.integers(1, 4))
        theta = rng.integers(-30, 30, size=8).astype(np.int8)
        comp = rng.integers(-64, 64, size=8).astype(np.int8)
        g = rng.integers(-2000, 2000, size=8).astype(np.int16)
        before = [Fr(int(t), 2 ** fl_in) + Fr(int(c), 2 ** (fl_in + d)) for t, c in zip(theta, comp)]
        steps = [Fr(frac_rne(-Fr(655, 2 ** 16) * Fr(int(x), 2 ** 12) * 2 ** (fl_in + d)), 2 ** (fl_in + d)) for x in g]
        ref.kahan_sgd_step(theta, comp, g, d, fl_in, fl_in + delta, 12, 655)
        fo = fl_in + delta
        for i in range(8):
            after = Fr(int(theta[i]), 2 ** fo) + Fr(int(comp[i]), 2 ** (fo + d))
            assert abs(after - (before[i] + steps[i])) <= Fr(1, 2 ** (fo + d + 1))


# ---- eq. 1 in fixed point: textbook round-then-clamp ---------------------------------------------------

def test_plain_sgd_is_round_half_even_then_clamp():
    rng = np.random.default_rng(6)
    for _ in range(300):
        fl_t, fl_g = int(rng.integers(-4, 12)), int(rng.integers(-4, 20))
        lr_q = int(rng.integers(1, 65536))
        theta = rng.integers(-128, 128, size=16).astype(np.int8)
        g = rng.integers(-32768, 32768, size=16).astype(np.int16)
        want = [max(-128, min(127, int(t) + round(-Fr(lr_q, 65536) * int(x) * Fr(2) ** (fl_t - fl_g))))
                for t, x in zip(theta, g)]
        ref.kahan_sgd_step(theta, None, g, 0, fl_t, fl_t, fl_g, lr_q)
        assert theta.tolist() == want


# ---- Section 1: uniform linear quantization, round-half-even, no stochastic rounding --------------------

@pytest.mark.parametrize("bits", [8, 16])
def test_quantize_matches_torch_round_clamp(bits):
    """For |x * 2^fl| < 2^23 the product is exact in fp32 and torch.round (half-to-even) then clamp is the definition."""
    g = torch.Generator().manual_seed(0)
    for fl in (-6, 0, 3, 7, 15, 22):
        x = torch.randn(4096, generator=g) * (2.0 ** (bits - 2 - fl))
        x[:64] = (torch.arange(64) - 32 + 0.5) * 2.0 ** (-fl)          # exact ties
        x = x[(x * 2.0 ** fl).abs() < 2 ** 23]
        want = torch.round(x * 2.0 ** fl).clamp(-(2 ** (bits - 1)), 2 ** (bits - 1) - 1).to(torch.int64)
        got = ref.quantize(x.numpy(), bits, fl)
        assert got.astype(np.int64).tolist() == want.tolist()


def test_quantize_hand_cases():
    f = np.float32
    # value in LSB units -> expected int8 code, fl = 4 (LSB = 1/16)
    cases = [(0.5, 0), (-0.5, 0), (1.5, 2), (-1.5, -2), (2.5, 2), (-2.5, -2), (126.5, 126), (127.5, 127),
             (127.49, 127), (-128.5, -128), (-129.0, -128), (1000.0, 127), (0.0, 0), (-0.0, 0)]
    x = np.array([v / 16.0 for v, _ in cases], dtype=f)
    st = ref.new_status()
    assert ref.quantize(x, 8, 4, st).tolist() == [w for _, w in cases] and st[0] == 0
    # subnormal input: exactly representable on a fine enough grid? 2^-149 * 2^64 is still tiny -> 0
    assert ref.quantize(np.array([1e-45, -1e-45], dtype=f), 16, 64).tolist() == [0, 0]
    # non-finite input
    st = ref.new_status()
    got = ref.quantize(np.array([np.nan, np.inf, -np.inf, 1.0], dtype=f), 16, 0, st)
    assert got.tolist() == [0, 32767, -32768, 1] and st[0] == ref.STATUS_NONFINITE
    # fraclen outside the domain: nothing written
    st = ref.new_status()
    out = np.full(2, 9, dtype=np.int8)
    ref.quantize(np.array([1.0, 2.0], dtype=f), 8, 65, st, out)
    assert out.tolist() == [9, 9] and st[0] == ref.STATUS_DOMAIN


# ---- Section 6: the exponent follows the tensor maximum -------------------------------------------------

def test_fraclen_hand_cases():
    f = np.float32
    sel = lambda M, W: ref.select_fraclen_f32(np.array([M / 4, -M, M / 2], dtype=f), W, 99)
    assert sel(0.5, 8) == 7            # 0.5 * 2^7 = 64; 2^8 would give 128 > 127
    assert sel(127.5, 8) == -1         # 127.5 rounds (half-even) to 128 at fl = 0
    assert sel(127.49, 8) == 0
    assert sel(1.0, 8) == 6 and sel(0.99, 8) == 7 and sel(0.999, 8) == 6     # 0.999*128 = 127.87 -> 128
    assert sel(1.0, 16) == 14
    assert sel(0.49999, 8) == 7        # 0.49999 * 256 = 127.997 would round to 128
    assert sel(1e-30, 16) == 64 and sel(3e38, 8) == -64                       # clamped to the domain
    assert ref.select_fraclen_f32(np.zeros(5, dtype=f), 8, 11) == 11          # all-zero tensor keeps the default
    assert ref.select_fraclen_f32(np.zeros(0, dtype=f), 8, 12) == 12
    st = ref.new_status()
    assert ref.select_fraclen_f32(np.array([1.0, np.nan], dtype=f), 8, 3, st) == -64 and st[0] == ref.STATUS_NONFINITE
    st = ref.new_status()
    assert ref.select_fraclen_f32(np.array([-np.inf, 1.0], dtype=f), 16, 3, st) == -64 and st[0] == ref.STATUS_NONFINITE


def test_reselect_widens_after_growth_with_one_step_lag():
    """A value that outgrows the grid saturates once, its excess lands in c, and the next grid is coarser."""
    theta, comp = one(120, np.int8), one(0, np.int8)
    grad = one(-32767, np.int16)
    fl_t, d = 7, 7
    # big step: lr ~ 1, g ~ -1.0 * 2^-... choose fl_g so that the step is +40 theta LSBs
    # step real = (65535/65536) * 32767 * 2^-fl_g ; want ~ 40 * 2^-7  ->  fl_g = 7 + 15 - 5.32 ~ 16.7 -> use 17
    vmax = ref.kahan_sgd_step(theta, comp, grad, d, fl_t, fl_t, 17, 65535)
    assert int(theta[0]) == 127                                   # saturated once
    v_real = Fr(vmax, 2 ** (fl_t + d))
    assert v_real > Fr(127, 2 ** fl_t)
    fl_next = ref.select_fraclen_vmax(vmax, fl_t + d, 8, fl_t)
    assert fl_next == fl_t - 1                                    # one bit coarser covers it
    # next step, no gradient: theta is re-expressed on the coarser grid, and theta + c is what is left
    before = Fr(int(theta[0]), 2 ** fl_t) + Fr(int(comp[0]), 2 ** (fl_t + d))
    ref.kahan_sgd_step(theta, comp, one(0, np.int16), d, fl_t, fl_next, 17, 65535)
    after = Fr(int(theta[0]), 2 ** fl_next) + Fr(int(comp[0]), 2 ** (fl_next + d))
    assert abs(after - before) <= Fr(1, 2 ** (fl_next + d + 1))
    assert abs(int(theta[0])) <= 64


def test_lr_constants_are_rne_of_the_decimal_literals():
    """Q0.16 learning rates used by the synthetic workloads (eta of eq. 1 as an unsigned 16-bit fraction)."""
    from decimal import Decimal
    for lit, q in (("0.01", 655), ("0.05", 3277), ("0.1", 6554), ("0.001", 66), ("0.0001", 7), ("0.5", 32768)):
        assert round(Fr(Decimal(lit)) * 2 ** 16) == q


# ---- Section 3, eq. 4-5: bit-width of the classifier from the class count -------------------------------

def test_classifier_bit_width_guideline():
    """What the paper states around eq. 5 with alpha = 0.5: 10-class tasks train with 8 bits everywhere, the 58-
    and 44-class transfer tasks use an 8-bit classifier, 1000-class ImageNet does not fit 8 bits and takes 16;
    plus the inequality of eq. 4 checked in exact rationals and eq. 5's closed form in floating point."""
    import math
    assert ref.classifier_min_bits(10) <= 8 and ref.classifier_min_bits(58) <= 8 and ref.classifier_min_bits(44) <= 8
    assert 8 < ref.classifier_min_bits(1000) <= 16
    assert [ref.classifier_min_bits(n) for n in (10, 58, 44, 1000)] == [6, 8, 8, 12]
    for n in (2, 3, 5, 9, 10, 17, 33, 100, 257, 1000, 21841, 1 << 20):
        for a_q in (32768, 1, 65535, 6554, 16384):
            bw = ref.classifier_min_bits(n, a_q)
            alpha = Fr(a_q, 65536)
            assert alpha / (n - 1) >= Fr(1, 2 ** (bw - 1))                      # eq. 4 holds at bw ...
            assert bw == 2 or alpha / (n - 1) < Fr(1, 2 ** (bw - 2))            # ... and fails one bit below
            bound = math.log2(n - 1) + math.log2(2 / float(alpha))              # eq. 5: bw > bound - (equality allowed by eq. 4)
            assert bw >= bound - 1e-9 and bw < bound + 1 + 1e-9 or bw == 2
    with pytest.raises(ValueError):
        ref.classifier_min_bits(1)
    with pytest.raises(ValueError):
        ref.classifier_min_bits(10, 0)

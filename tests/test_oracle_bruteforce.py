"""Oracle vs exact-rational brute force on tiny tensors (CPU only)."""
import random

import numpy as np
import pytest

from oracle import ref
import exact_rational as ex

DT = {8: np.int8, 16: np.int16}


def rand_q(rng, bits, extreme_p=0.25):
    lo, hi = -(2 ** (bits - 1)), 2 ** (bits - 1) - 1
    if rng.random() < extreme_p:
        return rng.choice([lo, hi, lo + 1, hi - 1, 0, 1, -1])
    return rng.randint(lo, hi)


def run_case(rng, tb, cb, gb, d, fl_in, delta, fl_g, lr_q, wd_q, kahan, n):
    fl_out = fl_in + delta
    theta = np.array([rand_q(rng, tb) for _ in range(n)], dtype=DT[tb])
    comp = np.array([rand_q(rng, cb) for _ in range(n)], dtype=DT[cb]) if kahan else None
    grad = np.array([rand_q(rng, gb) for _ in range(n)], dtype=DT[gb])
    want_t, want_c, want_v = [], [], 0
    for i in range(n):
        t, c, va = ex.step(int(theta[i]), int(comp[i]) if kahan else 0, int(grad[i]), tb, cb, d,
                           fl_in, fl_out, fl_g, lr_q, wd_q, kahan)
        want_t.append(t); want_c.append(c); want_v = max(want_v, va)
    st = ref.new_status()
    vmax = ref.kahan_sgd_step(theta, comp, grad, d, fl_in, fl_out, fl_g, lr_q, wd_q, st)
    ctx = dict(tb=tb, cb=cb, gb=gb, d=d, fl_in=fl_in, delta=delta, fl_g=fl_g, lr_q=lr_q, wd_q=wd_q, kahan=kahan)
    assert st[0] == 0, ctx
    assert theta.tolist() == want_t, ctx
    if kahan:
        assert comp.tolist() == want_c, ctx
    assert vmax == want_v, ctx


@pytest.mark.parametrize("seed", range(8))
def test_step_random_domain(seed):
    """All width combinations, random fraclens (negative shifts included), grid moves, decay, extremes."""
    rng = random.Random(1000 + seed)
    for _ in range(400):
        tb, cb, gb = rng.choice([8, 16]), rng.choice([8, 16]), rng.choice([8, 16])
        kahan = rng.random() < 0.85
        d = rng.choice([cb - 1, cb - 1, rng.randint(0, 24)])
        fl_in = rng.randint(-20, 30)
        delta = rng.choice([0, 0, 0, 1, -1, 2, -2, rng.randint(-15, 15)])
        # shift of the step = fl_g + 16 - (fl_in + d): cover multiply (<0), small and large divides
        k = rng.choice([rng.randint(-12, 0), rng.randint(1, 12), rng.randint(13, 34), rng.randint(-45, 50)])
        fl_g = k - 16 + fl_in + (d if kahan else 0)
        if not -64 <= fl_g <= 64:
            continue
        lr_q = rng.choice([1, 65535, 655, 32768, rng.randint(1, 65535)])
        wd_q = rng.choice([0, 0, 7, 65535, rng.randint(1, 65535)])
        run_case(rng, tb, cb, gb, d, fl_in, delta, fl_g, lr_q, wd_q, kahan, rng.randint(1, 8))


def test_step_typical_shifts():
    """The shifts the synthetic workloads actually produce (step shift 9..31, default d, no grid move)."""
    rng = random.Random(7)
    for _ in range(1500):
        tb = rng.choice([8, 16]); cb = tb; d = cb - 1
        fl_in = rng.randint(0, 16)
        k = rng.randint(9, 33)
        fl_g = k - 16 + fl_in + d
        run_case(rng, tb, cb, 16, d, fl_in, 0, fl_g, rng.choice([655, 3277, 6554, 66, rng.randint(1, 65535)]),
                 rng.choice([0, 7]), True, 8)


def test_step_saturation_and_cap():
    """Drive theta' and c' into both rails; exercise the 2^40 cap with a gradient grid far coarser than c's."""
    rng = random.Random(11)
    hit_cap = 0
    for _ in range(600):
        tb, cb = rng.choice([8, 16]), rng.choice([8, 16])
        d = cb - 1
        fl_in = rng.randint(-5, 20)
        k = rng.randint(-45, -8)                     # multiply by 2^8..2^45
        fl_g = k - 16 + fl_in + d
        if fl_g < -64:
            continue
        if -k + 16 > 40:
            hit_cap += 1
        run_case(rng, tb, cb, 16, d, fl_in, rng.choice([0, -3, 3]), fl_g, rng.choice([65535, 30000]), 0, True, 6)
    assert hit_cap > 50


def test_out_of_domain_leaves_tensor_untouched():
    theta = np.array([5, -7], dtype=np.int8); comp = np.array([1, 2], dtype=np.int8)
    grad = np.array([100, -100], dtype=np.int16)
    for kw in (dict(fl_in=65, fl_out=64, fl_g=0, d=7), dict(fl_in=0, fl_out=16, fl_g=0, d=7),
               dict(fl_in=0, fl_out=0, fl_g=-65, d=7), dict(fl_in=0, fl_out=0, fl_g=0, d=25)):
        st = ref.new_status()
        t, c = theta.copy(), comp.copy()
        v = ref.kahan_sgd_step(t, c, grad, kw["d"], kw["fl_in"], kw["fl_out"], kw["fl_g"], 655, 0, st)
        assert st[0] == ref.STATUS_DOMAIN and v == 0
        assert (t == theta).all() and (c == comp).all()


@pytest.mark.parametrize("bits", [8, 16])
def test_quantize_bruteforce(bits):
    rng = np.random.default_rng(5)
    for _ in range(300):
        fl = int(rng.integers(-64, 65))
        # values near the grid, near ties, near saturation, tiny, huge
        scale = 2.0 ** (-fl)
        base = rng.integers(-2 ** (bits - 1) - 3, 2 ** (bits - 1) + 3, size=6).astype(np.float64)
        off = rng.choice([0.0, 0.5, -0.5, 0.25, 0.499999, 0.500001], size=6)
        x = ((base + off) * scale).astype(np.float32)
        x = np.concatenate([x, rng.standard_normal(4).astype(np.float32) * np.float32(scale * 2 ** (bits - 2)),
                            np.array([0.0, -0.0, 1e-45, -1e-45, 3e38, -3e38], dtype=np.float32)])
        st = ref.new_status()
        got = ref.quantize(x, bits, fl, st)
        assert st[0] == 0
        assert got.tolist() == [ex.quantize(v, bits, fl) for v in x], (bits, fl)


@pytest.mark.parametrize("bits", [8, 16])
def test_fraclen_is_largest_non_saturating(bits):
    rng = np.random.default_rng(9)
    pats = rng.integers(1, 0x7F800000, size=250, dtype=np.int64)
    # significands just below a power of two, where rounding tips the maximum over the rail
    edge = []
    for e in range(60, 200, 7):
        for m in (0x7FFFFF, 0x7FFFFF - (1 << (23 - bits)), 0x800000 - (1 << (24 - bits)) - 0x800000 & 0x7FFFFF,
                  0x7FFFFF - (1 << (24 - bits)) + 1, 0x7FFFFF - (1 << (24 - bits)), 0):
            edge.append((e << 23) | (m & 0x7FFFFF))
    pats = np.concatenate([pats, np.array(edge, dtype=np.int64)]).astype(np.uint32)
    for p in pats:
        M = np.array([p], dtype=np.uint32).view(np.float32)
        x = np.array([0.0, -M[0], M[0] / 3], dtype=np.float32)
        fl = ref.select_fraclen_f32(x, bits, 99)
        Mf = ex.f32_to_fraction(M[0])
        assert fl == ex.fraclen(Mf, bits), (hex(int(p)), bits)
        if -64 < fl < 64:
            assert ex.passes(Mf, bits, fl) and not ex.passes(Mf, bits, fl + 1)
            # quantizing a tensor with its own fraclen never saturates
            q = ref.quantize(x, bits, fl)
            assert abs(int(q[1])) == ex.rne(Mf * ex.two(fl)) <= 2 ** (bits - 1) - 1


@pytest.mark.parametrize("bits", [8, 16])
def test_fraclen_from_vmax_bruteforce(bits):
    rng = random.Random(13)
    from fractions import Fraction as Fr
    for _ in range(400):
        vmax = rng.choice([1, 2, 127, 128, 255, 32767, 32768, rng.randint(1, 2 ** 42), (1 << rng.randint(1, 41)) - 1,
                           ((1 << bits) - 1) << rng.randint(0, 20), (((1 << bits) - 1) << rng.randint(1, 20)) - 1])
        F = rng.randint(-40, 88)
        cur = rng.randint(max(-64, F - 24), min(64, F))
        fl = ref.select_fraclen_vmax(vmax, F, bits, cur)
        want = ex.fraclen(Fr(vmax) * ex.two(-F), bits)
        want = max(cur - 15, min(cur + 15, want))
        want = max(-64, min(64, want))
        assert fl == want, (vmax, F, bits, cur)
    assert ref.select_fraclen_vmax(0, 10, bits, 5) == 5

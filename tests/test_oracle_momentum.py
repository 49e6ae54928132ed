"""Oracle of momentum SGD with the lazy update inside: exact-rational brute force and closed-form pins (CPU only)."""
import random
from fractions import Fraction as Fr

import numpy as np
import pytest

from oracle import ref
import exact_rational as ex

DT = {8: np.int8, 16: np.int16}


def rand_q(rng, bits):
    lo, hi = -(2 ** (bits - 1)), 2 ** (bits - 1) - 1
    return rng.choice([lo, hi, 0, 1, -1, rng.randint(lo, hi), rng.randint(lo, hi), rng.randint(-9, 9)])


@pytest.mark.parametrize("seed", range(6))
def test_momentum_step_bruteforce(seed):
    rng = random.Random(300 + seed)
    done = 0
    while done < 300:
        tb, cb, mb, gb = (rng.choice([8, 16]) for _ in range(4))
        kahan = rng.random() < 0.85
        d = rng.choice([cb - 1, cb - 1, rng.randint(0, 24)]) if kahan else 0
        fl_in = rng.randint(-15, 25)
        delta = rng.choice([0, 0, 0, 1, -1, rng.randint(-15, 15)])
        fl_m_in = fl_in + rng.randint(-6, 22)
        delta_m = rng.choice([0, 0, 0, 1, -2, rng.randint(-15, 15)])
        fl_m_out = fl_m_in + delta_m
        fl_g = fl_m_out + rng.choice([rng.randint(0, 12), rng.randint(-20, 30), rng.randint(-50, 60)])
        if not all(-64 <= f <= 64 for f in (fl_in, fl_in + delta, fl_m_in, fl_m_out, fl_g)):
            continue
        lr_q = rng.choice([1, 65535, 655, 6554, rng.randint(1, 65535)])
        mu_q = rng.choice([0, 58982, 65535, 32768, rng.randint(0, 65535)])
        wd_q = rng.choice([0, 0, 7, 65535])
        n = rng.randint(1, 6)
        theta = np.array([rand_q(rng, tb) for _ in range(n)], dtype=DT[tb])
        comp = np.array([rand_q(rng, cb) for _ in range(n)], dtype=DT[cb]) if kahan else None
        mom = np.array([rand_q(rng, mb) for _ in range(n)], dtype=DT[mb])
        grad = np.array([rand_q(rng, gb) for _ in range(n)], dtype=DT[gb])
        want = [ex.momentum_step(int(theta[i]), int(comp[i]) if kahan else 0, int(mom[i]), int(grad[i]), tb, cb, mb, d,
                                 fl_in, fl_in + delta, fl_m_in, fl_m_out, fl_g, lr_q, mu_q, wd_q, kahan) for i in range(n)]
        st = ref.new_status()
        vmax, mmax = ref.momentum_sgd_step(theta, comp, mom, grad, d, fl_in, fl_in + delta, fl_m_in, fl_m_out, fl_g,
                                           lr_q, mu_q, wd_q, st)
        ctx = dict(tb=tb, cb=cb, mb=mb, gb=gb, d=d, fl=(fl_in, delta, fl_m_in, fl_m_out, fl_g), lr=lr_q, mu=mu_q, wd=wd_q)
        assert st[0] == 0, ctx
        assert theta.tolist() == [w[0] for w in want], ctx
        if kahan:
            assert comp.tolist() == [w[1] for w in want], ctx
        assert mom.tolist() == [w[2] for w in want], ctx
        assert vmax == max(w[3] for w in want) and mmax == max(w[4] for w in want), ctx
        done += 1


def test_zero_momentum_on_a_shared_grid_is_the_plain_lazy_update():
    """mu = 0 and a velocity wide and fine enough to hold the step exactly (int16 velocity on c's grid, step
    below 2^15 c-LSBs and a gradient grid that needs no rounding): the velocity equals the step of Algorithm 1
    and theta, c follow the non-momentum update bit for bit."""
    rng = np.random.default_rng(1)
    for _ in range(100):
        fl_t, d = int(rng.integers(0, 10)), 7
        F = fl_t + d
        fl_g = F - 16 + int(rng.integers(0, 3))         # -lr_q*g lands on c's grid after dividing by 2^(0..2) ...
        lr_q = 1 << int(rng.integers(2, 6))             # ... exactly, because lr_q is a multiple of 4
        n = 32
        theta = rng.integers(-100, 100, size=n).astype(np.int8); comp = rng.integers(-60, 60, size=n).astype(np.int8)
        g = rng.integers(-400, 400, size=n).astype(np.int16)
        t2, c2 = theta.copy(), comp.copy()
        mom = rng.integers(-30000, 30000, size=n).astype(np.int16)      # ignored: mu = 0
        v1 = ref.kahan_sgd_step(theta, comp, g, d, fl_t, fl_t, fl_g, lr_q)
        v2, _ = ref.momentum_sgd_step(t2, c2, mom, g, d, fl_t, fl_t, F, F, fl_g, lr_q, 0)
        assert np.array_equal(theta, t2) and np.array_equal(comp, c2) and v1 == v2
        want_m = [-(lr_q * int(x)) // (1 << (fl_g + 16 - F)) for x in g]          # exact division by construction
        assert mom.tolist() == want_m


def test_velocity_decay_and_fixed_point():
    """No gradient: the velocity follows m <- round_half_even(mu * m) (Python's own rounding on Fractions) and
    stalls where rounding wins over decay (|m| <= 4 for mu = 0.9) -- the known low-precision plateau.
    Constant gradient: it climbs to the fixed point of m = round(mu * m + step)."""
    mu_q = 58982                                   # RNE(0.9 * 65536)
    for m0 in (127, -128, 50, -7, 5, 4, 1, 0):
        mom = np.array([m0], dtype=np.int8); theta = np.zeros(1, dtype=np.int8); comp = np.zeros(1, dtype=np.int8)
        g = np.zeros(1, dtype=np.int16)
        m = m0
        for _ in range(60):
            ref.momentum_sgd_step(theta, comp, mom, g, 7, 7, 7, 12, 12, 20, 655, mu_q)
            m = max(-128, min(127, round(Fr(mu_q, 65536) * m)))
            assert int(mom[0]) == m
        assert abs(m) <= 4 and (abs(m0) <= 4) == (m == m0)      # 0.9 * 5 = 4.5 - eps rounds down, 0.9 * 4 = 3.6 rounds back up
    # constant step of exactly 3 velocity LSBs per update: fl_g + 16 - (fl_m + 16) = 4, lr_q * |g| = 3 * 2^16 * 2^4
    mom = np.zeros(1, dtype=np.int8); theta = np.zeros(1, dtype=np.int8); comp = np.zeros(1, dtype=np.int8)
    g = np.array([-96], dtype=np.int16)             # 32768 * 96 = 3 * 2^20
    m, hist = 0, []
    for _ in range(80):
        ref.momentum_sgd_step(theta, comp, mom, g, 7, 7, 7, 12, 12, 16, 32768, mu_q)
        m = max(-128, min(127, round(Fr(mu_q, 65536) * m + 3)))
        assert int(mom[0]) == m
        hist.append(m)
    assert hist[-1] == hist[-2] and 25 <= hist[-1] <= 30            # 3 / (1 - 0.9) = 30, minus the rounding plateau


def test_momentum_conserves_theta_plus_c():
    """The lazy update inside still conserves: theta*2^d + c grows by exactly the quantized velocity each step."""
    rng = np.random.default_rng(2)
    n, d, fl_t, fl_m, fl_g = 48, 7, 6, 17, 20
    theta = rng.integers(-40, 40, size=n).astype(np.int8); comp = np.zeros(n, dtype=np.int8)
    mom = np.zeros(n, dtype=np.int8)
    total = [int(t) << d for t in theta]
    for step in range(200):
        g = rng.integers(-2500, 2500, size=n).astype(np.int16)
        vmax, _ = ref.momentum_sgd_step(theta, comp, mom, g, d, fl_t, fl_t, fl_m, fl_m, fl_g, 6554, 58982)
        for i in range(n):
            total[i] += round(Fr(int(mom[i])) * Fr(2) ** (fl_t + d - fl_m))       # the new velocity, on c's grid
            assert (int(theta[i]) << d) + int(comp[i]) == total[i]
        assert vmax == max(abs(v) for v in total)
    assert np.abs(theta.astype(int)).max() < 127


def test_momentum_out_of_domain():
    theta = np.array([1], dtype=np.int8); comp = np.array([2], dtype=np.int8); mom = np.array([3], dtype=np.int8)
    g = np.array([4], dtype=np.int16)
    for kw in (dict(fl_m_in=65), dict(fl_m_out=-65), dict(fl_m_in=0, fl_m_out=16), dict(fl_out=30)):
        a = dict(fl_in=7, fl_out=7, fl_m_in=10, fl_m_out=10, fl_g=12); a.update(kw)
        st = ref.new_status()
        assert ref.momentum_sgd_step(theta, comp, mom, g, 7, a["fl_in"], a["fl_out"], a["fl_m_in"], a["fl_m_out"], a["fl_g"],
                                     655, 58982, 0, st) == (0, 0)
        assert st[0] == ref.STATUS_DOMAIN and (int(theta[0]), int(comp[0]), int(mom[0])) == (1, 2, 3)

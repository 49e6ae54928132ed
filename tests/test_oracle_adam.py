"""Oracle of ADAM with the lazy update inside (Section 4: ADAM in INT16, Algorithm 1 in the optimizer): exact-rational
brute force, the optimizer's textbook properties and a float64 cross-check (CPU only)."""
import math
import random
from fractions import Fraction as Fr

import numpy as np
import pytest

from oracle import ref
import exact_rational as ex

DT = {8: np.int8, 16: np.int16}
B1, B2 = 58982, 65470            # RNE(0.9 * 2^16), RNE(0.999 * 2^16)


def rand_q(rng, bits):
    lo, hi = -(2 ** (bits - 1)), 2 ** (bits - 1) - 1
    return rng.choice([lo, hi, 0, 1, -1, rng.randint(lo, hi), rng.randint(lo, hi), rng.randint(-9, 9)])


def domain_e(fl_in, d, fl_u_out, lr_exp, fl_m_out):
    R = (fl_u_out + 24 + fl_u_out % 2) // 2
    return fl_in + d + R - 16 - lr_exp - fl_m_out


@pytest.mark.parametrize("seed", range(6))
def test_adam_step_bruteforce(seed):
    rng = random.Random(700 + seed)
    done = 0
    while done < 250:
        tb, cb, mb, ub, gb = (rng.choice([8, 16]) for _ in range(5))
        kahan = rng.random() < 0.85
        d = rng.choice([cb - 1, cb - 1, rng.randint(0, 24)]) if kahan else 0
        fl_in = rng.randint(-10, 25)
        delta = rng.choice([0, 0, 0, 1, -1, rng.randint(-15, 15)])
        fl_g = rng.randint(-5, 40)
        fl_m_in = fl_g + rng.choice([0, 1, -1, rng.randint(-12, 12)])
        fl_m_out = fl_m_in + rng.choice([0, 0, 0, 1, -2, rng.randint(-15, 15)])
        fl_u_in = 2 * fl_g + rng.choice([0, 1, -1, rng.randint(-20, 10), rng.randint(-40, 30)])
        fl_u_out = fl_u_in + rng.choice([0, 0, 0, 1, -1, rng.randint(-15, 15)])
        lr_exp = rng.choice([0, 0, 3, 10, rng.randint(0, 48)])
        eps_q, eps_exp = rng.choice([(0, 0), (43980, 26), (65535, 0), (1, 48), (rng.randint(0, 65535), rng.randint(0, 48))])
        if not all(-64 <= f <= 64 for f in (fl_in, fl_in + delta, fl_m_in, fl_m_out, fl_u_in, fl_u_out, fl_g)):
            continue
        if domain_e(fl_in, d, fl_u_out, lr_exp, fl_m_out) > 20:
            continue
        lr_q = rng.choice([1, 65535, 66, 6554, rng.randint(1, 65535)])
        b1_q = rng.choice([B1, 32768, 0, 65535, rng.randint(0, 65535)])
        b2_q = rng.choice([B2, 58982, 0, 65535, rng.randint(0, 65535)])
        n = rng.randint(1, 6)
        theta = np.array([rand_q(rng, tb) for _ in range(n)], dtype=DT[tb])
        comp = np.array([rand_q(rng, cb) for _ in range(n)], dtype=DT[cb]) if kahan else None
        mom = np.array([rand_q(rng, mb) for _ in range(n)], dtype=DT[mb])
        sec = np.array([rng.choice([abs(rand_q(rng, ub)) % 2 ** (ub - 1), rand_q(rng, ub)]) for _ in range(n)], dtype=DT[ub])
        grad = np.array([rand_q(rng, gb) for _ in range(n)], dtype=DT[gb])
        want = [ex.adam_step(int(theta[i]), int(comp[i]) if kahan else 0, int(mom[i]), int(sec[i]), int(grad[i]),
                             tb, cb, mb, ub, d, fl_in, fl_in + delta, fl_m_in, fl_m_out, fl_u_in, fl_u_out, fl_g,
                             lr_q, lr_exp, b1_q, b2_q, eps_q, eps_exp, kahan) for i in range(n)]
        st = ref.new_status()
        vmax, mmax, umax = ref.adam_step(theta, comp, mom, sec, grad, d, fl_in, fl_in + delta, fl_m_in, fl_m_out,
                                         fl_u_in, fl_u_out, fl_g, lr_q, lr_exp, b1_q, b2_q, eps_q, eps_exp, st)
        ctx = dict(w=(tb, cb, mb, ub, gb), d=d, fl=(fl_in, delta, fl_m_in, fl_m_out, fl_u_in, fl_u_out, fl_g),
                   lr=(lr_q, lr_exp), b=(b1_q, b2_q), eps=(eps_q, eps_exp))
        assert st[0] == 0, ctx
        assert theta.tolist() == [w[0] for w in want], ctx
        if kahan:
            assert comp.tolist() == [w[1] for w in want], ctx
        assert mom.tolist() == [w[2] for w in want], ctx
        assert sec.tolist() == [w[3] for w in want], ctx
        assert (vmax, mmax, umax) == (max(w[4] for w in want), max(w[5] for w in want), max(w[6] for w in want)), ctx
        done += 1


def lr_pair(lr):
    """lr = lr_q * 2^-(16 + lr_exp) with the largest exponent that keeps lr_q in 16 bits."""
    e = 0
    while e < 48 and lr * 2.0 ** (16 + e + 1) <= 65535:
        e += 1
    return int(round(lr * 2.0 ** (16 + e))), e


def test_constant_gradient_moves_theta_by_lr_per_step():
    """Textbook property: with the bias corrections in the step size and eps -> 0, a constant gradient gives
    m_t / sqrt(u_t) = sign(g) at every t, so every step has size lr whatever the gradient's scale.  Here in int16
    throughout (theta with a 16-bit accumulator, d = 15): the virtual parameter theta + c moves by lr per step to
    within the 16-bit resolution of the two moments."""
    lr = 1e-3
    for gval, fl_g in ((12000, 20), (-3, 3), (32767, 30)):
        theta = np.zeros(4, dtype=np.int16); comp = np.zeros(4, dtype=np.int16)
        mom = np.zeros(4, dtype=np.int16); sec = np.zeros(4, dtype=np.int16)
        g = np.full(4, gval, dtype=np.int16)
        fl_t, d = 14, 15
        # grids of the moments: the finest that hold |g| and g^2
        fl_m = fl_g + (15 - int(math.floor(math.log2(abs(gval)))) - 1)
        fl_u = 2 * fl_g + (15 - int(math.floor(math.log2(gval * gval))) - 1)
        steps = 60
        for t in range(1, steps + 1):
            lr_t = lr * math.sqrt(1 - (B2 / 65536) ** t) / (1 - (B1 / 65536) ** t)
            lr_q, lr_exp = lr_pair(lr_t)
            ref.adam_step(theta, comp, mom, sec, g, d, fl_t, fl_t, fl_m, fl_m, fl_u, fl_u, fl_g, lr_q, lr_exp, B1, B2, 0, 0)
            virt = (int(theta[0]) * 2 ** d + int(comp[0])) * 2.0 ** -(fl_t + d)
            want = -math.copysign(lr * t, gval)
            assert abs(virt - want) <= 0.03 * lr * t + 2.0 ** -(fl_t + d), (gval, t, virt, want)
        assert len(set(theta.tolist())) == 1 and int(mom[0]) * gval > 0 and int(sec[0]) > 0


def test_step_is_invariant_to_the_gradient_scale():
    """ADAM's step does not depend on the scale of the gradients (eps = 0): moving the gradient grid by k bits and
    the grids of the two moments by k and 2k leaves every stored integer and every step exactly as it was."""
    rng = np.random.default_rng(5)
    n = 64
    base = None
    for k in (0, 3, -4, 7):
        r = np.random.default_rng(9)
        theta = r.integers(-100, 100, size=n).astype(np.int8); comp = np.zeros(n, dtype=np.int8)
        mom = np.zeros(n, dtype=np.int16); sec = np.zeros(n, dtype=np.int16)
        fl_g, fl_m, fl_u = 20 + k, 22 + k, 34 + 2 * k
        hist = []
        for t in range(25):
            g = r.integers(-20000, 20000, size=n).astype(np.int16)
            out = ref.adam_step(theta, comp, mom, sec, g, 7, 6, 6, fl_m, fl_m, fl_u, fl_u, fl_g, 40000, 5, B1, B2, 0, 0)
            hist.append((theta.copy(), comp.copy(), mom.copy(), sec.copy(), out))
        if base is None:
            base = hist
        else:
            for a, b in zip(base, hist):
                assert all(np.array_equal(x, y) for x, y in zip(a[:4], b[:4])) and a[4] == b[4]
    assert rng is not None


def test_against_float64_adam():
    """A few hundred steps of random gradients in wide formats (int16 theta + int16 accumulator, int16 moments)
    stay close to ADAM in float64 with the same hyper-parameters: the fixed-point rule is the textbook one.
    The second moment grows a thousandfold while its bias decays (beta2 = 0.999), so its grid follows its
    running maximum from step to step (dynamic fixed point, one bit of headroom for the one-step lag)."""
    rng = np.random.default_rng(11)
    n, steps, lr, eps = 256, 300, 2e-3, 1e-4      # eps well above the 16-bit floor of sqrt(u): no early blow-up
    fl_t, d, fl_g, fl_m = 14, 15, 24, 23
    b1, b2 = B1 / 65536, B2 / 65536
    theta = np.zeros(n, dtype=np.int16); comp = np.zeros(n, dtype=np.int16)
    mom = np.zeros(n, dtype=np.int16); sec = np.zeros(n, dtype=np.int16)
    mean = rng.normal(0, 5e-4, size=n)
    tf, mf, uf = np.zeros(n), np.zeros(n), np.zeros(n)
    eps_q, eps_exp = lr_pair(eps)
    fl_u_in = fl_u_out = 42                                # (1 - beta2) g^2 of the first step fits
    fl_u_seen = set()
    for t in range(1, steps + 1):
        greal = mean + rng.normal(0, 5e-4, size=n)
        g = np.clip(np.rint(greal * 2.0 ** fl_g), -32768, 32767).astype(np.int16)
        gq = g.astype(np.float64) * 2.0 ** -fl_g
        lr_t = lr * math.sqrt(1 - b2 ** t) / (1 - b1 ** t)
        lr_q, lr_exp = lr_pair(lr_t)
        _, _, umax = ref.adam_step(theta, comp, mom, sec, g, d, fl_t, fl_t, fl_m, fl_m, fl_u_in, fl_u_out, fl_g,
                                   lr_q, lr_exp, B1, B2, eps_q, eps_exp)
        assert umax <= 32767                                # the headroom was enough: nothing saturated
        fl_u_seen.add(fl_u_out)
        fl_u_in, fl_u_out = fl_u_out, ref.select_fraclen_vmax(umax, fl_u_out, 16, fl_u_out) - 1
        mf = b1 * mf + (1 - b1) * gq
        uf = b2 * uf + (1 - b2) * gq * gq
        tf = tf - lr_t * mf / (np.sqrt(uf) + eps)
    virt = (theta.astype(np.float64) * 2.0 ** d + comp) * 2.0 ** -(fl_t + d)
    assert len(fl_u_seen) >= 6                                                # the grid really followed the growth
    assert np.abs(tf).max() > 0.05                                            # the run really moved
    assert np.abs(virt - tf).max() <= 0.01 * np.abs(tf).max()
    assert np.corrcoef(virt, tf)[0, 1] > 0.9999
    assert np.abs(mom * 2.0 ** -fl_m - mf).max() <= 0.01 * np.abs(mf).max()
    assert np.abs(sec * 2.0 ** -fl_u_in - uf).max() <= 0.01 * np.abs(uf).max()


def test_second_moment_needs_16_bits():
    """Section 4: "INT16 was necessary for the ADAM optimizer because of beta2 (= 0.999)".  With an 8-bit second
    moment the decay (1 - beta2) u is below half an LSB for every representable u, so u can never come down: after
    the gradients vanish it stays where it was, while a 16-bit one decays."""
    for bits, moves in ((8, False), (16, True)):
        sec = np.array([2 ** (bits - 1) - 1 - 20], dtype=DT[bits]); u0 = int(sec[0])
        theta = np.zeros(1, dtype=np.int8); comp = np.zeros(1, dtype=np.int8); mom = np.zeros(1, dtype=np.int16)
        g = np.zeros(1, dtype=np.int16)
        for _ in range(200):
            ref.adam_step(theta, comp, mom, sec, g, 7, 7, 7, 20, 20, 30, 30, 20, 66, 0, B1, B2, 0, 0)
        assert (int(sec[0]) < u0) == moves, (bits, int(sec[0]))
        if moves:
            assert abs(int(sec[0]) - u0 * (B2 / 65536) ** 200) <= 0.02 * u0


def test_adam_out_of_domain_and_bad_arguments():
    theta = np.array([1], dtype=np.int8); comp = np.array([2], dtype=np.int8); mom = np.array([3], dtype=np.int16)
    sec = np.array([5], dtype=np.int16); g = np.array([4], dtype=np.int16)
    base = dict(fl_in=7, fl_out=7, fl_m_in=10, fl_m_out=10, fl_u_in=20, fl_u_out=20, fl_g=12)
    for kw in (dict(fl_u_in=65), dict(fl_u_out=-65), dict(fl_u_in=0, fl_u_out=16), dict(fl_m_out=30), dict(fl_out=30),
               dict(fl_in=40, fl_out=40, fl_m_in=-20, fl_m_out=-20, fl_u_in=60, fl_u_out=60)):   # the last: e = 73 > 20
        a = dict(base); a.update(kw)
        st = ref.new_status()
        out = ref.adam_step(theta, comp, mom, sec, g, 7, a["fl_in"], a["fl_out"], a["fl_m_in"], a["fl_m_out"], a["fl_u_in"],
                            a["fl_u_out"], a["fl_g"], 655, 0, B1, B2, 0, 0, st)
        assert out == (0, 0, 0) and st[0] == ref.STATUS_DOMAIN
        assert (int(theta[0]), int(comp[0]), int(mom[0]), int(sec[0])) == (1, 2, 3, 5)
    for bad in (dict(lr_q=65536), dict(lr_exp=49), dict(b1_q=70000), dict(eps_exp=49)):
        a = dict(lr_q=655, lr_exp=0, b1_q=B1, b2_q=B2, eps_q=0, eps_exp=0); a.update(bad)
        with pytest.raises(Exception):
            ref.adam_step(theta, comp, mom, sec, g, 7, 7, 7, 10, 10, 20, 20, 12, a["lr_q"], a["lr_exp"], a["b1_q"], a["b2_q"],
                          a["eps_q"], a["eps_exp"])

"""Exact-rational restatement of the lazy update, for tiny inputs.

Every quantity is a `fractions.Fraction` of the REAL numbers the fixed-point
words stand for (theta * 2^-fl etc.); nothing here shifts integers.  It is the
brute-force checker the CPU oracle is pinned against: written from the update
rule of Algorithm 1 (Section 2) in real-number terms, with its own
round-half-even.
"""
from fractions import Fraction as Fr

CAP = 2 ** 40


def two(e):
    return Fr(2) ** e


def rne(x):
    """Round a Fraction to the nearest integer, ties to the even one."""
    x = Fr(x)
    lo = x.numerator // x.denominator          # floor
    frac = x - lo
    if frac > Fr(1, 2):
        return lo + 1
    if frac < Fr(1, 2):
        return lo
    return lo if lo % 2 == 0 else lo + 1


def sat(q, bits):
    return max(-(2 ** (bits - 1)), min(2 ** (bits - 1) - 1, q))


def f32_to_fraction(x):
    """Exact value of a finite numpy float32."""
    return Fr(float(x))          # float32 -> float64 is exact, Fraction(float) is exact


def quantize(x, bits, fl):
    return sat(rne(f32_to_fraction(x) * two(fl)), bits)


def passes(M, bits, fl):
    """Does the magnitude M (a Fraction) fit a `bits`-wide grid of fraclen fl without saturating?"""
    return rne(M * two(fl)) <= 2 ** (bits - 1) - 1


def fraclen(M, bits, lo=-64, hi=64):
    """Largest fl at which M does not saturate, by exhaustive search, then clamped."""
    assert M > 0
    best = None
    for fl in range(-420, 421):
        if passes(M, bits, fl):
            best = fl
    return max(lo, min(hi, best))


def _apply(theta, c, s, theta_bits, comp_bits, d, fl_in, fl_out, kahan):
    """Fold an already quantized step s (an integer number of c-LSBs of the input grid) into theta and c."""
    F = fl_in + d
    v_real = theta * two(-fl_in) + c * two(-F) + s * two(-F)      # the compensated sum, kept wide
    theta_new = sat(rne(v_real * two(fl_out)), theta_bits)
    resid = v_real - theta_new * two(-fl_out)
    c_new = sat(rne(resid * two(fl_out + d)), comp_bits) if kahan else 0
    vabs = abs(v_real) * two(F)
    assert vabs.denominator == 1
    return theta_new, c_new, int(vabs)


def step(theta, c, g, theta_bits, comp_bits, d, fl_in, fl_out, fl_g, lr_q, wd_q=0, kahan=True):
    """One element.  Returns (theta', c', |v| in units of the working grid)."""
    if not kahan:
        d, c = 0, 0
    F = fl_in + d                                  # grid of the compensation word
    lr, wd = Fr(lr_q, 2 ** 16), Fr(wd_q, 2 ** 16)
    theta_real, g_real = theta * two(-fl_in), g * two(-fl_g)
    s = max(-CAP, min(CAP, rne(-lr * g_real * two(F))))
    if wd_q:
        s += max(-CAP, min(CAP, rne(-lr * wd * theta_real * two(F))))
    return _apply(theta, c, s, theta_bits, comp_bits, d, fl_in, fl_out, kahan)


def momentum_step(theta, c, m, g, theta_bits, comp_bits, mom_bits, d, fl_in, fl_out, fl_m_in, fl_m_out, fl_g,
                  lr_q, mu_q, wd_q=0, kahan=True):
    """Momentum SGD (velocity m <- mu*m - lr*(g + wd*theta), theta <- theta + m) with the lazy update inside.
    Returns (theta', c', m', |v| on grid F, |velocity before saturation| on grid fl_m_out)."""
    if not kahan:
        d, c = 0, 0
    lr, mu, wd = Fr(lr_q, 2 ** 16), Fr(mu_q, 2 ** 16), Fr(wd_q, 2 ** 16)
    G = fl_m_out + 16
    w = rne(mu * m * two(-fl_m_in) * two(G))
    w += max(-CAP, min(CAP, rne(-lr * g * two(-fl_g) * two(G))))
    if wd_q:
        w += max(-CAP, min(CAP, rne(-lr * wd * theta * two(-fl_in) * two(G))))
    m_wide = rne(Fr(w, 2 ** 16))
    m_new = sat(m_wide, mom_bits)
    F = fl_in + d
    s = max(-CAP, min(CAP, rne(m_new * two(-fl_m_out) * two(F))))
    t, cn, vabs = _apply(theta, c, s, theta_bits, comp_bits, d, fl_in, fl_out, kahan)
    return t, cn, m_new, vabs, abs(m_wide)


def adam_step(theta, c, m, u, g, theta_bits, comp_bits, mom_bits, sec_bits, d, fl_in, fl_out, fl_m_in, fl_m_out,
              fl_u_in, fl_u_out, fl_g, lr_q, lr_exp, b1_q, b2_q, eps_q, eps_exp, kahan=True):
    """ADAM (m <- b1 m + (1-b1) g, u <- b2 u + (1-b2) g^2, theta <- theta - lr_t m / (sqrt(u) + eps)) with the lazy
    update inside, in real-number terms.  The root is taken on the grid R = (fl_u_out + 24 + parity) / 2 and
    checked here by its defining inequality.  Returns (theta', c', m', u', |v| on grid F, |m| and max(u, 0)
    before saturation)."""
    import math
    if not kahan:
        d, c = 0, 0
    b1, b2 = Fr(b1_q, 2 ** 16), Fr(b2_q, 2 ** 16)
    lr_t, eps = Fr(lr_q) * two(-(16 + lr_exp)), Fr(eps_q) * two(-(16 + eps_exp))
    g_real = g * two(-fl_g)
    Gm, Gu = fl_m_out + 16, fl_u_out + 16
    wM = rne(b1 * m * two(-fl_m_in) * two(Gm)) + max(-CAP, min(CAP, rne((1 - b1) * g_real * two(Gm))))
    m_wide = rne(Fr(wM, 2 ** 16))
    m_new = sat(m_wide, mom_bits)
    wU = rne(b2 * u * two(-fl_u_in) * two(Gu)) + max(-CAP, min(CAP, rne((1 - b2) * g_real * g_real * two(Gu))))
    u_wide = rne(Fr(wU, 2 ** 16))
    u_new = max(0, min(2 ** (sec_bits - 1) - 1, u_wide))
    par = fl_u_out % 2                                  # Python's % is already the non-negative parity
    R = Fr(fl_u_out + 24 + par, 2)
    assert R.denominator == 1
    R = int(R)
    x = u_new * two(-fl_u_out) * two(2 * R)             # the radicand on grid 2R: an integer
    assert x.denominator == 1
    rt = math.isqrt(int(x))
    assert Fr(rt * rt) <= x < Fr((rt + 1) * (rt + 1))   # rt * 2^-R <= sqrt(u') < (rt + 1) * 2^-R
    den = max(rt + min(rne(eps * two(R)), 2 ** 30), 1)
    F = fl_in + d
    s = max(-CAP, min(CAP, rne(-lr_t * m_new * two(-fl_m_out) / (den * two(-R)) * two(F))))
    t, cn, vabs = _apply(theta, c, s, theta_bits, comp_bits, d, fl_in, fl_out, kahan)
    return t, cn, m_new, u_new, vabs, abs(m_wide), max(u_wide, 0)

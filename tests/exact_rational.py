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


def step(theta, c, g, theta_bits, comp_bits, d, fl_in, fl_out, fl_g, lr_q, wd_q=0, kahan=True):
    """One element.  Returns (theta', c', |v| in units of the working grid)."""
    if not kahan:
        d, c = 0, 0
    F = fl_in + d                                  # grid of the compensation word
    lr, wd = Fr(lr_q, 2 ** 16), Fr(wd_q, 2 ** 16)
    theta_real, c_real, g_real = theta * two(-fl_in), c * two(-F), g * two(-fl_g)

    s = max(-CAP, min(CAP, rne(-lr * g_real * two(F))))
    if wd_q:
        s += max(-CAP, min(CAP, rne(-lr * wd * theta_real * two(F))))
    v_real = theta_real + c_real + s * two(-F)      # the compensated sum, kept wide

    theta_new = sat(rne(v_real * two(fl_out)), theta_bits)
    resid = v_real - theta_new * two(-fl_out)
    c_new = sat(rne(resid * two(fl_out + d)), comp_bits) if kahan else 0
    vabs = abs(v_real) * two(F)
    assert vabs.denominator == 1
    return theta_new, c_new, int(vabs)

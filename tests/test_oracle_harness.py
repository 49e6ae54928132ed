"""The threaded front ends of the oracle (harness conveniences for large tensors) return exactly what the single C
routine returns on the whole array."""
import numpy as np
import pytest

from oracle import ref


@pytest.mark.parametrize("bits", [8, 16])
def test_threaded_fraclen_selection_equals_the_single_scan(bits):
    rng = np.random.default_rng(5)
    for trial in range(60):
        n = int(rng.integers(1, 5000))
        x = (rng.standard_normal(n) * 10.0 ** rng.uniform(-8, 6)).astype(np.float32)
        kind = trial % 6
        if kind == 1:
            x[: n // 2] = 0.0                                  # all-zero chunks next to live ones
        elif kind == 2:
            x[:] = 0.0                                         # all zero: the default comes back
        elif kind == 3:
            x[int(rng.integers(0, n))] = np.float32(np.nan)
        elif kind == 4:
            x[int(rng.integers(0, n))] = np.float32(-np.inf)
        elif kind == 5:
            x[int(rng.integers(0, n))] = np.float32(2.0 ** int(rng.integers(-20, 20)) * (1 - 2.0 ** -bits))   # near a rail
        for dflt in (-3, 7, 15):
            sa, sb = ref.new_status(), ref.new_status()
            a = ref.select_fraclen_f32(x, bits, dflt, sa)
            b = ref.select_fraclen_f32_mt(x, bits, dflt, sb, threads=4, chunk=int(rng.integers(1, 700)))
            assert a == b and int(sa[0]) == int(sb[0]), (trial, kind, dflt, a, b)


def test_threaded_quantize_and_step_equal_the_single_call():
    rng = np.random.default_rng(9)
    n = 10007
    x = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    fl = ref.select_fraclen_f32(x, 16, 15)
    g1, g2 = ref.quantize(x, 16, fl), ref.quantize_mt(x, 16, fl, threads=4, chunk=999)
    assert np.array_equal(g1, g2)
    th = rng.integers(-128, 128, n).astype(np.int8)
    co = rng.integers(-128, 128, n).astype(np.int8)
    t1, c1, t2, c2 = th.copy(), co.copy(), th.copy(), co.copy()
    v1 = ref.kahan_sgd_step(t1, c1, g1, 7, 7, 7, fl, 6554, 7)
    v2 = ref.kahan_sgd_step_mt(t2, c2, g1, 7, 7, 7, fl, 6554, 7, threads=4, chunk=1234)
    assert v1 == v2 and np.array_equal(t1, t2) and np.array_equal(c1, c2)

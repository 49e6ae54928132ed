"""The update kernels fed from the fp32 gradients (`*_f32grad`: quantization in registers) on random multi-tensor
lists, against the oracle's quantize followed by its update (needs an MI355X): every width combination, comp shifts,
grid moves, misaligned buffers, ragged sizes, gradients on and beyond the rails of their grid, rounding ties, and now
and then a NaN or an infinity.  LPK_FUZZ_SEEDS=lo:hi runs more seeds."""
import os
import random
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

from oracle import ref
from paper_1810_05486_amd import binding as lpk

NP = {8: np.int8, 16: np.int16}
TT = {8: torch.int8, 16: torch.int16}
DEV = "cuda:0"
SIZES = [0, 1, 15, 16, 17, 255, 1024, 4095, 4096, 4097, 9001, 33000]


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def fuzz_seeds(default_count):
    spec = os.environ.get("LPK_FUZZ_SEEDS")
    if not spec:
        return range(default_count)
    lo, hi = (int(x) for x in spec.split(":"))
    return range(lo, hi)


def fp32_gradients(rng, n, gb, fl_g, special):
    """fp32 values whose images on the DFX(gb, fl_g) grid cover the whole code range and a little beyond it, sitting
    on grid points, a quarter and (almost) a half LSB off them, and exactly on ties; with `special`, a NaN and both
    infinities somewhere."""
    lim = 2 ** (gb - 1)
    q = rng.integers(-lim - 3, lim + 3, size=n).astype(np.float64)
    q += rng.choice([0.0, 0.0, 0.25, -0.25, 0.5, -0.5, 0.49, -0.49], size=n)
    x = (q * 2.0 ** (-fl_g)).astype(np.float32)              # exact: at most 19 significant bits times a power of two
    if special and n >= 8:
        x[rng.integers(0, n)] = np.nan
        x[rng.integers(0, n)] = np.inf
        x[rng.integers(0, n)] = -np.inf
    return x


def make_case(rng, pr, widths, fls, d, n=None, mis=None, special=None):
    """widths = (tb, cb, mb, ub, gb) with 0 for an absent array; fls: the fraclens the call will get, fl_g last."""
    tb, cb, mb, ub, gb = widths
    n = pr.choice(SIZES) if n is None else n
    mis = pr.choice([0, 0, 0, 1, 8, 16]) if mis is None else mis
    c = dict(n=n, widths=widths, fls=list(fls), d=d, mis=mis)
    c["theta"] = rng.integers(-(2 ** (tb - 1)), 2 ** (tb - 1), size=n).astype(NP[tb])
    c["comp"] = rng.integers(-(2 ** (cb - 1)), 2 ** (cb - 1), size=n).astype(NP[cb]) if cb else None
    c["mom"] = rng.integers(-(2 ** (mb - 1)), 2 ** (mb - 1), size=n).astype(NP[mb]) if mb else None
    c["sec"] = rng.integers(0, pr.choice([4, 300, 2 ** (ub - 1)]), size=n).astype(NP[ub]) if ub else None
    c["src"] = fp32_gradients(rng, n, gb, fls[-1], special=pr.random() < 0.15 if special is None else special)
    c["bufs"] = []

    def dev(a, dtype):
        buf = torch.zeros(n + 64, dtype=dtype, device=DEV)
        v = buf[mis:mis + n]
        v.copy_(torch.from_numpy(a))
        c["bufs"].append(buf)
        return v
    c["d_theta"] = dev(c["theta"], TT[tb])
    c["d_comp"] = dev(c["comp"], TT[cb]) if cb else None
    c["d_mom"] = dev(c["mom"], TT[mb]) if mb else None
    c["d_sec"] = dev(c["sec"], TT[ub]) if ub else None
    c["d_src"] = dev(c["src"], torch.float32)
    c["grad_sentinel"] = np.full(n, 77, dtype=NP[gb])       # the int gradient array: named by the descriptor, never touched
    c["d_grad"] = dev(c["grad_sentinel"], TT[gb])
    return c


def descriptor(c):
    shift = c["d"] if c["widths"][1] and c["d"] is not None else lpk.LPK_COMP_SHIFT_DEFAULT
    return lpk.make_desc(c["d_theta"], c["d_comp"], c["d_grad"], c["d_src"], shift, momentum=c["d_mom"], second=c["d_sec"])


def check(cases, call, oracle_step, n_max):
    """Run `call(list, fraclen arrays, maxima, status)`, then the oracle's quantize + `oracle_step` tensor by tensor."""
    tl = lpk.TensorList([descriptor(c) for c in cases])
    if sum(c["n"] for c in cases) % 3 == 0:                  # a third of the lists with every store forced
        lpk.lpk_tensor_list_set_option(tl, lpk.LPK_OPT_STORE_ALL, 1)
    i32 = dict(dtype=torch.int32, device=DEV)
    arr = [torch.tensor([c["fls"][j] for c in cases], **i32) for j in range(len(cases[0]["fls"]))]
    mx = [torch.full((len(cases),), 5 + k, dtype=torch.int64, device=DEV) for k in range(n_max)]
    status = torch.zeros(1, **i32)
    call(tl, arr, mx, status)
    torch.cuda.synchronize()
    st = ref.new_status()
    for i, c in enumerate(cases):
        tb, cb, mb, ub, gb = c["widths"]
        dd = c["d"] if c["d"] is not None else (cb - 1 if cb else 0)
        g = ref.quantize(c["src"], gb, c["fls"][-1], st)
        want = oracle_step(c, g, dd, st)
        ctx = dict(i=i, n=c["n"], widths=c["widths"], d=dd, fls=c["fls"], mis=c["mis"])
        for key in ("theta", "comp", "mom", "sec"):
            if c[key] is not None:
                assert np.array_equal(c["d_" + key].cpu().numpy(), c[key]), (key, ctx)
        assert np.array_equal(c["d_grad"].cpu().numpy(), c["grad_sentinel"]), ("int gradient array written", ctx)
        assert tuple(int(m[i].item()) for m in mx) == tuple(want), ("maxima", ctx)
        for b in c["bufs"]:                                  # guard words behind every (possibly shifted) view
            assert int(b[-8:].abs().sum().item()) == 0, ("guard", ctx)
    assert int(status.cpu().numpy().view(np.uint32)[0]) == int(st[0])
    tl.destroy()


def clamp_fl(f):
    return max(-64, min(64, f))


@pytest.mark.parametrize("seed", fuzz_seeds(3))
def test_fused_plain_update_random_lists(seed):
    say("fused plain update: random lists, seed %d" % seed)
    rng = np.random.default_rng(2100 + seed)
    pr = random.Random(2200 + seed)
    for rep in range(6):
        cases = []
        for _ in range(pr.randint(1, 10)):
            tb, gb = pr.choice([8, 16]), pr.choice([16, 16, 8])
            cb = pr.choice([8, 16, tb, tb, 0])
            d = pr.choice([None, None, pr.randint(0, 24)]) if cb else None
            dd = d if d is not None else (cb - 1 if cb else 0)
            fl_in = pr.randint(-20, 30)
            delta = pr.choice([0, 0, 0, 1, -1, 3, -4, pr.randint(-15, 15)])
            k = pr.choice([pr.randint(9, 33), pr.randint(9, 33), pr.randint(1, 8), pr.randint(-30, 0), pr.randint(30, 60)])
            fls = [clamp_fl(fl_in), clamp_fl(fl_in + delta), clamp_fl(k - 16 + fl_in + dd)]
            cases.append(make_case(rng, pr, (tb, cb, 0, 0, gb), fls, d))
        lr_q, wd_q = pr.choice([1, 655, 6554, 32768, 65535]), pr.choice([0, 0, 7, 65535])

        def call(tl, arr, mx, status):
            lpk.lpk_kahan_sgd_step_f32grad(tl, arr[0], arr[1], arr[2], lr_q, wd_q, mx[0], status)

        def oracle_step(c, g, dd, st):
            f = c["fls"]
            return (ref.kahan_sgd_step(c["theta"], c["comp"], g, dd, f[0], f[1], f[2], lr_q, wd_q, st),)
        check(cases, call, oracle_step, 1)


@pytest.mark.parametrize("seed", fuzz_seeds(3))
def test_fused_momentum_update_random_lists(seed):
    say("fused momentum update: random lists, seed %d" % seed)
    rng = np.random.default_rng(2300 + seed)
    pr = random.Random(2400 + seed)
    for rep in range(6):
        cases = []
        for _ in range(pr.randint(1, 10)):
            tb, mb = pr.choice([8, 16]), pr.choice([8, 16])
            cb = pr.choice([tb, tb, tb, 8, 16, 0])
            gb = pr.choice([16, 16, 16, 8])
            d = pr.choice([None, None, pr.randint(0, 24)]) if cb else None
            dd = d if d is not None else (cb - 1 if cb else 0)
            fl_in = pr.randint(-10, 20)
            delta = pr.choice([0, 0, 0, 0, 1, -1, pr.randint(-15, 15)])
            fl_m_in = fl_in + dd + pr.randint(-8, 12)
            fl_m_out = fl_m_in + pr.choice([0, 0, 0, 0, 1, -1, pr.randint(-15, 15)])
            fl_g = fl_m_out + pr.choice([pr.randint(1, 14), pr.randint(1, 14), pr.randint(-20, 0), pr.randint(15, 50)])
            fls = [clamp_fl(f) for f in (fl_in, fl_in + delta, fl_m_in, fl_m_out, fl_g)]
            cases.append(make_case(rng, pr, (tb, cb, mb, 0, gb), fls, d))
        lr_q, mu_q, wd_q = pr.choice([1, 655, 6554, 65535]), pr.choice([58982, 32768, 0, 65535]), pr.choice([0, 0, 7, 65535])

        def call(tl, arr, mx, status):
            lpk.lpk_momentum_sgd_step_f32grad(tl, arr[0], arr[1], arr[2], arr[3], arr[4], lr_q, mu_q, wd_q, mx[0], mx[1], status)

        def oracle_step(c, g, dd, st):
            f = c["fls"]
            return ref.momentum_sgd_step(c["theta"], c["comp"], c["mom"], g, dd, f[0], f[1], f[2], f[3], f[4], lr_q, mu_q, wd_q, st)
        check(cases, call, oracle_step, 2)


@pytest.mark.parametrize("seed", fuzz_seeds(3))
def test_fused_adam_update_random_lists(seed):
    say("fused adam update: random lists, seed %d" % seed)
    rng = np.random.default_rng(2500 + seed)
    pr = random.Random(2600 + seed)
    for rep in range(6):
        cases = []
        standing = pr.random() < 0.4               # lists on which the kernel's short arithmetic route applies
        for _ in range(pr.randint(1, 10)):
            tb = pr.choice([8, 16])
            mb, ub = (16, 16) if standing else pr.choice([(16, 16), (16, 16), (16, 16), (8, 16), (16, 8), (8, 8)])
            cb = pr.choice([tb, tb, tb, 8, 16, 0])
            gb = pr.choice([16, 16, 16, 8])
            d = pr.choice([None, None, pr.randint(0, 24)]) if cb else None
            fl_in = pr.randint(-10, 20)
            delta = 0 if standing else pr.choice([0, 0, 0, 0, 1, -1, pr.randint(-15, 15)])
            fl_g = pr.randint(0, 40)
            fl_m_in = fl_g + (pr.choice([0, 1, 2, 8, 9]) if standing else pr.choice([0, 1, -1, pr.randint(-12, 12)]))
            fl_m_out = fl_m_in + (0 if standing else pr.choice([0, 0, 0, 0, 1, -1, pr.randint(-15, 15)]))
            fl_u_in = 2 * fl_g + (pr.choice([-7, -8, -11, -6]) if standing else pr.choice([0, -3, pr.randint(-25, 8), pr.randint(-40, 30)]))
            fl_u_out = fl_u_in + (0 if standing else pr.choice([0, 0, 0, 0, 1, -1, pr.randint(-15, 15)]))
            fls = [clamp_fl(f) for f in (fl_in, fl_in + delta, fl_m_in, fl_m_out, fl_u_in, fl_u_out, fl_g)]
            cases.append(make_case(rng, pr, (tb, cb, mb, ub, gb), fls, d))
        hyper = (pr.choice([1, 66, 21000, 65535]), pr.choice([0, 0, 4, 11, pr.randint(0, 48)]),
                 pr.choice([58982, 32768, 0, 65535]), pr.choice([65470, 58982, 0, 65535]),
                 pr.choice([0, 43980, 65535, 1]), pr.choice([0, 26, 10, pr.randint(0, 48)]))

        def call(tl, arr, mx, status):
            lpk.lpk_adam_step_f32grad(tl, arr[0], arr[1], arr[2], arr[3], arr[4], arr[5], arr[6], hyper, mx[0], mx[1], mx[2], status)

        def oracle_step(c, g, dd, st):
            f = c["fls"]
            return ref.adam_step(c["theta"], c["comp"], c["mom"], c["sec"], g, dd, f[0], f[1], f[2], f[3], f[4], f[5], f[6],
                                 *hyper, status=st)
        check(cases, call, oracle_step, 3)


@pytest.mark.parametrize("kernel", ["plain", "momentum", "adam"])
def test_a_tensor_skipped_for_its_domain_still_reports_non_finite_gradients(kernel):
    """The fused calls stand for quantize-then-update, status word included.  A tensor whose parameter fraclens are
    out of range is skipped untouched, but the quantization would have looked at its gradients: a NaN among them
    raises the non-finite bit next to the domain bit.  With the gradients' own fraclen out of range the quantization
    would have skipped the tensor too, and only the domain bit is raised."""
    say("fused %s: skipped tensor with a NaN among its gradients" % kernel)
    rng = np.random.default_rng(7)
    pr = random.Random(7)
    widths = {"plain": (8, 8, 0, 0, 16), "momentum": (8, 8, 16, 0, 16), "adam": (8, 8, 16, 16, 16)}[kernel]
    n_fl = {"plain": 3, "momentum": 5, "adam": 7}[kernel]
    for fl_g, want_status in ((20, lpk.LPK_STATUS_DOMAIN | lpk.LPK_STATUS_NONFINITE), (99, lpk.LPK_STATUS_DOMAIN)):
        good = [7, 7, 21, 21, 33, 33, 20]
        fls_good = good[:n_fl - 1] + [20]
        fls_bad = [7, 7 + 16] + good[2:n_fl - 1] + [fl_g]            # theta's grid moves by 16 > 15: outside the domain
        a = make_case(rng, pr, widths, fls_good, None, n=5000, mis=0, special=False)
        b = make_case(rng, pr, widths, fls_bad, None, n=9000, mis=0, special=False)
        b["src"][4321] = np.nan
        b["d_src"].copy_(torch.from_numpy(b["src"]))
        before = {k: b[k].copy() for k in ("theta", "comp", "mom", "sec") if b[k] is not None}
        hyper = (66, 0, 58982, 65470, 43980, 26)

        def call(tl, arr, mx, status):
            if kernel == "plain":
                lpk.lpk_kahan_sgd_step_f32grad(tl, arr[0], arr[1], arr[2], 655, 0, mx[0], status)
            elif kernel == "momentum":
                lpk.lpk_momentum_sgd_step_f32grad(tl, arr[0], arr[1], arr[2], arr[3], arr[4], 655, 58982, 0, mx[0], mx[1], status)
            else:
                lpk.lpk_adam_step_f32grad(tl, arr[0], arr[1], arr[2], arr[3], arr[4], arr[5], arr[6], hyper, mx[0], mx[1], mx[2], status)

        def oracle_step(c, g, dd, st):
            f = c["fls"]
            if kernel == "plain":
                return (ref.kahan_sgd_step(c["theta"], c["comp"], g, dd, f[0], f[1], f[2], 655, 0, st),)
            if kernel == "momentum":
                return ref.momentum_sgd_step(c["theta"], c["comp"], c["mom"], g, dd, f[0], f[1], f[2], f[3], f[4], 655, 58982, 0, st)
            return ref.adam_step(c["theta"], c["comp"], c["mom"], c["sec"], g, dd, *f, *hyper, status=st)
        tl = lpk.TensorList([descriptor(a), descriptor(b)])
        status = torch.zeros(1, dtype=torch.int32, device=DEV)
        arr = [torch.tensor([a["fls"][j], b["fls"][j]], dtype=torch.int32, device=DEV) for j in range(n_fl)]
        mx = [torch.full((2,), 9, dtype=torch.int64, device=DEV) for _ in range(3)]
        call(tl, arr, mx, status)
        torch.cuda.synchronize()
        assert int(status.cpu().numpy().view(np.uint32)[0]) == want_status, (kernel, fl_g)
        for k, v in before.items():
            assert np.array_equal(b["d_" + k].cpu().numpy(), v), (kernel, fl_g, k, "skipped tensor written")
        tl.destroy()
        if fl_g > 64:
            continue
        # and the whole list against the oracle's quantize + update, status word included
        a2 = make_case(rng, pr, widths, fls_good, None, n=5000, mis=0, special=False)
        b2 = make_case(rng, pr, widths, fls_bad, None, n=9000, mis=0, special=False)
        b2["src"][17] = np.inf
        b2["d_src"].copy_(torch.from_numpy(b2["src"]))
        check([a2, b2], call, oracle_step, {"plain": 1, "momentum": 2, "adam": 3}[kernel])

"""GPU library vs CPU oracle on edge cases, through the C ABI (needs an MI355X): ragged and empty tensors,
unaligned pointers, every width combination, grid moves, negative shifts, rails, the boundaries between the
kernel's 32-bit and 64-bit arithmetic paths, special fp32 values, and the status word."""
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


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def fuzz_seeds(default_count):
    """Seeds of the random-list tests: 0..default_count-1, or LPK_FUZZ_SEEDS=lo:hi for a longer differential run."""
    import os
    spec = os.environ.get("LPK_FUZZ_SEEDS")
    if not spec:
        return range(default_count)
    lo, hi = (int(x) for x in spec.split(":"))
    return range(lo, hi)


class Case:
    """One tensor of a list: host copies for the oracle, device copies (possibly misaligned views) for the library."""

    def __init__(self, rng, n, tb, cb, gb, d, fl_in, fl_out, fl_g, misalign=0, g_lim=None, th_lim=None):
        self.n, self.tb, self.cb, self.gb, self.d = n, tb, cb, gb, d
        self.fl_in, self.fl_out, self.fl_g = fl_in, fl_out, fl_g
        lo_t, hi_t = (-(2 ** (tb - 1)), 2 ** (tb - 1)) if th_lim is None else (-th_lim, th_lim)
        lo_g, hi_g = (-(2 ** (gb - 1)), 2 ** (gb - 1)) if g_lim is None else (-g_lim, g_lim)
        self.theta = rng.integers(lo_t, hi_t, size=n).astype(NP[tb])
        self.comp = rng.integers(-(2 ** (cb - 1)), 2 ** (cb - 1), size=n).astype(NP[cb]) if cb else None
        self.grad = rng.integers(lo_g, hi_g, size=n).astype(NP[gb])
        if n >= 4:                      # plant the extremes
            self.grad[0], self.grad[1] = -(2 ** (gb - 1)), 2 ** (gb - 1) - 1
            self.theta[2], self.theta[3] = -(2 ** (tb - 1)), 2 ** (tb - 1) - 1

        def dev(a, bits):
            buf = torch.zeros(n + 64, dtype=TT[bits], device=DEV)        # base is 256-byte aligned
            v = buf[misalign:misalign + n]
            v.copy_(torch.from_numpy(a))
            return buf, v

        self.keep = []
        self.d_theta = self.d_comp = None
        b, self.d_theta = dev(self.theta, tb); self.keep.append(b)
        if cb:
            b, self.d_comp = dev(self.comp, cb); self.keep.append(b)
        b, self.d_grad = dev(self.grad, gb); self.keep.append(b)

    def desc(self):
        return lpk.make_desc(self.d_theta, self.d_comp, self.d_grad, None,
                             self.d if self.cb and self.d is not None else lpk.LPK_COMP_SHIFT_DEFAULT)


def run_list(cases, lr_q, wd_q, want_vmax=True, store_all=False):
    tl = lpk.TensorList([c.desc() for c in cases])
    if store_all:
        lpk.lpk_tensor_list_set_option(tl, lpk.LPK_OPT_STORE_ALL, 1)
    i32 = dict(dtype=torch.int32, device=DEV)
    fl_in = torch.tensor([c.fl_in for c in cases], **i32)
    fl_out = torch.tensor([c.fl_out for c in cases], **i32)
    fl_g = torch.tensor([c.fl_g for c in cases], **i32)
    vmax = torch.full((len(cases),), 77, dtype=torch.int64, device=DEV)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    lpk.lpk_kahan_sgd_step(tl, fl_in, fl_out, fl_g, lr_q, wd_q, vmax if want_vmax else None, status)
    torch.cuda.synchronize()
    st = ref.new_status()
    for i, c in enumerate(cases):
        d = c.d if c.d is not None else (c.cb - 1 if c.cb else 0)
        want_v = ref.kahan_sgd_step(c.theta, c.comp, c.grad, d, c.fl_in, c.fl_out, c.fl_g, lr_q, wd_q, st)
        ctx = dict(i=i, n=c.n, tb=c.tb, cb=c.cb, gb=c.gb, d=d, fl=(c.fl_in, c.fl_out, c.fl_g), lr=lr_q, wd=wd_q)
        assert np.array_equal(c.d_theta.cpu().numpy(), c.theta), ("theta", ctx)
        if c.cb:
            assert np.array_equal(c.d_comp.cpu().numpy(), c.comp), ("comp", ctx)
        if want_vmax:
            assert int(vmax[i].item()) == want_v, ("vmax", ctx)
        # guard words around a misaligned view stay untouched
        for b in c.keep:
            assert int(b[-8:].abs().sum().item()) == 0
    assert int(status.cpu().numpy().view(np.uint32)[0]) == int(st[0])
    tl.destroy()
    return int(st[0])


SIZES = [0, 1, 15, 16, 17, 63, 64, 255, 1023, 1024, 1025, 4095, 4096, 4097, 8191, 12289, 70001]


@pytest.mark.parametrize("seed", fuzz_seeds(6))
def test_random_lists_all_widths_shifts_and_alignments(seed):
    say("random multi-tensor lists, seed %d" % seed)
    rng = np.random.default_rng(100 + seed)
    pr = random.Random(200 + seed)
    for rep in range(6):
        cases = []
        for _ in range(pr.randint(1, 12)):
            tb, gb = pr.choice([8, 16]), pr.choice([16, 16, 8])
            cb = pr.choice([8, 16, tb, tb, 0])
            d = pr.choice([None, None, pr.randint(0, 24)]) if cb else None
            dd = d if d is not None else (cb - 1 if cb else 0)
            fl_in = pr.randint(-20, 30)
            delta = pr.choice([0, 0, 0, 1, -1, 3, -4, pr.randint(-15, 15)])
            k = pr.choice([pr.randint(9, 33), pr.randint(9, 33), pr.randint(1, 8), pr.randint(-30, 0), pr.randint(30, 60)])
            fl_g = max(-64, min(64, k - 16 + fl_in + dd))
            fl_out = max(-64, min(64, fl_in + delta))
            cases.append(Case(rng, pr.choice(SIZES), tb, cb, gb, d, fl_in, fl_out, fl_g,
                              misalign=pr.choice([0, 0, 0, 1, 3, 8, 16])))
        run_list(cases, pr.choice([1, 655, 6554, 32768, 65535]), pr.choice([0, 0, 7, 65535]),
                 want_vmax=pr.random() < 0.8, store_all=pr.random() < 0.3)


@pytest.mark.parametrize("tb", [8, 16])
def test_arithmetic_path_boundaries(tb):
    """Shifts on both sides of every condition that selects the 32-bit path (step shift 8|9, d 0|1, widest d
    that still fits, extreme lr and gradients, decay on/off) and its FMA-rounding variant for small values
    (d 8|9, step bound either side of 2^22), same-width aligned tensors of several tiles."""
    say("path boundaries, %d-bit" % tb)
    rng = np.random.default_rng(tb)
    for kg in (8, 9, 10, 23, 31, 32, 33, 48, 90):
        for d in (0, 1, tb - 1, 8, 9, 15, 16, 22, 24):
            fl_in = 5
            fl_g = kg - 16 + fl_in + d
            if not -64 <= fl_g <= 64:
                continue
            cases = [Case(rng, 9000 + 13, tb, tb, 16, d, fl_in, fl_in, fl_g)]
            for lr_q, wd_q in ((65535, 0), (1, 0), (6554, 7), (65535, 65535)):
                run_list(cases, lr_q, wd_q)


def test_rails_are_hit_in_the_vector_path():
    """A large constant step drives theta and comp into both rails over a few steps."""
    say("saturation in the vector path")
    rng = np.random.default_rng(3)
    c = Case(rng, 3 * 4096 + 5, 8, 8, 16, None, 7, 7, 10)      # step shift 12: up to 4096 theta LSBs per step
    hit = 0
    for _ in range(3):
        run_list([c], 65535, 0)
        hit += int((np.abs(c.theta.astype(np.int32)) >= 127).sum())
    assert hit > 1000


def test_out_of_domain_tensor_is_skipped_and_flagged():
    say("domain status")
    rng = np.random.default_rng(4)
    good = Case(rng, 5000, 8, 8, 16, None, 7, 7, 20)
    bad1 = Case(rng, 5000, 8, 8, 16, None, 7, 23, 20)          # grid move of 16
    bad2 = Case(rng, 300, 16, 16, 16, None, 65, 65, 20)        # fraclen outside [-64, 64]
    bad3 = Case(rng, 300, 8, 0, 16, None, 0, 0, -70)
    assert run_list([good, bad1, bad2, bad3], 655, 0) == lpk.LPK_STATUS_DOMAIN


def _select_quantize(xs, bits_sel, theta_bits=8):
    """Run select(F32) + quantize through the library on a list of fp32 arrays; return (fl list, q list, status)."""
    n_t = len(xs)
    src = [torch.from_numpy(x.copy()).to(DEV) for x in xs]
    theta = [torch.zeros(max(x.size, 1), dtype=TT[theta_bits], device=DEV)[:x.size] for x in xs]
    grad = [torch.zeros(max(x.size, 1), dtype=torch.int16, device=DEV)[:x.size] for x in xs]
    descs = []
    for t in range(n_t):
        d = lpk.make_desc(theta[t], None, grad[t], src[t])
        descs.append(d)
    tl = lpk.TensorList(descs)
    fl = torch.tensor([40 + t for t in range(n_t)], dtype=torch.int32, device=DEV)     # defaults, recognisable
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    lpk.lpk_select_fraclen(tl, lpk.LPK_F32, bits_sel, None, None, fl, fl, status)
    lpk.lpk_quantize_tensor(tl, bits_sel, fl, status)
    torch.cuda.synchronize()
    out = theta if bits_sel == lpk.LPK_SEL_THETA else grad
    res = ([int(v) for v in fl.cpu()], [o.cpu().numpy() for o in out], int(status.cpu().numpy().view(np.uint32)[0]))
    tl.destroy()
    return res


@pytest.mark.parametrize("sel,bits", [(lpk.LPK_SEL_GRAD, 16), (lpk.LPK_SEL_THETA, 8), (lpk.LPK_SEL_THETA, 16)])
def test_select_and_quantize_special_values(sel, bits):
    say("select + quantize special values, %d-bit" % bits)
    f = np.float32
    rng = np.random.default_rng(8)
    xs = [
        np.zeros(100, dtype=f),                                           # all zero -> default fraclen
        np.array([], dtype=f),                                            # empty -> default
        np.array([0.0, -0.0, 1e-45, -1e-45, 1e-40], dtype=f),             # subnormals only -> clamped to 64
        np.array([1.0, np.nan, -2.0], dtype=f),
        np.array([np.inf, 1.0], dtype=f),
        np.array([-np.inf], dtype=f),
        np.array([3e38, -1e38], dtype=f),                                 # clamps to -64, saturates
        np.array([0.5, -0.25, 0.125], dtype=f),
        np.array([127.5, -3.0], dtype=f), np.array([127.49, 2.0], dtype=f),
        np.array([0.49999, 0.1], dtype=f), np.array([0.999, -0.998], dtype=f),
        (rng.standard_normal(4096 * 3 + 7) * 1e-3).astype(f),
        (rng.standard_normal(17) * 1e5).astype(f),
        np.array([(i - 40 + 0.5) / 64.0 for i in range(80)], dtype=f),    # exact ties at the chosen grid
    ]
    # significands around the rounding edge of the fraclen rule
    for m in (0x7FFFFF, 0x7FFFFF - (1 << (24 - bits)) + 1, 0x7FFFFF - (1 << (24 - bits)), 0x7F0000):
        xs.append(np.array([(100 << 23) | m, (90 << 23) | 5], dtype=np.uint32).view(f).copy())
    fls, qs, status = _select_quantize(xs, sel, theta_bits=bits if sel == lpk.LPK_SEL_THETA else 8)
    st = ref.new_status()
    for t, x in enumerate(xs):
        want_fl = ref.select_fraclen_f32(x, bits, 40 + t, st)
        assert fls[t] == want_fl, (t, fls[t], want_fl)
        want_q = ref.quantize(x, bits, want_fl, st)
        assert np.array_equal(qs[t], want_q), (t, x[:8], qs[t][:8], want_q[:8])
    assert status == int(st[0]) == ref.STATUS_NONFINITE


def test_quantize_every_fraclen_and_domain_flag():
    say("quantize across the fraclen domain")
    rng = np.random.default_rng(9)
    base = np.concatenate([rng.standard_normal(1000).astype(np.float32),
                           np.array([0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 32767.5, -32768.5, 1e15, -1e15], dtype=np.float32)])
    fls = list(range(-64, 65, 4)) + [-64, 64, 65, -65, 1000]
    xs = [(base * np.float32(2.0) ** np.float32(-min(max(fl, -60), 60))).astype(np.float32) for fl in fls]
    src = [torch.from_numpy(x).to(DEV) for x in xs]
    grad = [torch.full((x.size,), 9, dtype=torch.int16, device=DEV) for x in xs]
    theta = [torch.zeros(x.size, dtype=torch.int8, device=DEV) for x in xs]
    tl = lpk.TensorList([lpk.make_desc(theta[t], None, grad[t], src[t]) for t in range(len(xs))])
    fl = torch.tensor(fls, dtype=torch.int32, device=DEV)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    lpk.lpk_quantize_tensor(tl, lpk.LPK_SEL_GRAD, fl, status)
    torch.cuda.synchronize()
    st = ref.new_status()
    for t, x in enumerate(xs):
        want = np.full(x.size, 9, dtype=np.int16)
        ref.quantize(x, 16, fls[t], st, out=want)
        assert np.array_equal(grad[t].cpu().numpy(), want), fls[t]
    assert int(status.cpu().numpy().view(np.uint32)[0]) == int(st[0]) == ref.STATUS_DOMAIN
    tl.destroy()


def test_reselect_from_vmax_matches_oracle():
    say("fraclen re-selection from vmax")
    pr = random.Random(5)
    n_t = 500
    theta = torch.zeros(16, dtype=torch.int8, device=DEV)
    theta16 = torch.zeros(16, dtype=torch.int16, device=DEV)
    comp = torch.zeros(16, dtype=torch.int8, device=DEV)
    comp16 = torch.zeros(16, dtype=torch.int16, device=DEV)
    grad = torch.zeros(16, dtype=torch.int16, device=DEV)
    descs, meta = [], []
    for t in range(n_t):
        tb = pr.choice([8, 16]); has_c = pr.random() < 0.8
        d = pr.choice([7, 15, pr.randint(0, 24)]) if has_c else 0
        descs.append(lpk.make_desc(theta if tb == 8 else theta16, (comp if pr.random() < .5 else comp16) if has_c else None,
                                   grad, None, d if has_c else lpk.LPK_COMP_SHIFT_DEFAULT))
        meta.append((tb, d))
    tl = lpk.TensorList(descs)
    vm, fin, cur = [], [], []
    for t in range(n_t):
        tb, d = meta[t]
        vm.append(pr.choice([0, 1, 127, 128, 255, 256, (1 << pr.randint(1, 45)) - 1, pr.randint(1, 1 << 42),
                             ((1 << tb) - 1) << pr.randint(0, 25), (((1 << tb) - 1) << pr.randint(1, 25)) - 1]))
        fi = pr.randint(-64, 64) if pr.random() < .95 else pr.choice([-70, 70])
        fin.append(fi)
        cur.append(max(-64, min(64, fi + pr.randint(-15, 15))) if pr.random() < .97 else 80)
    d_vm = torch.tensor(vm, dtype=torch.int64, device=DEV)
    d_fin = torch.tensor(fin, dtype=torch.int32, device=DEV)
    d_cur = torch.tensor(cur, dtype=torch.int32, device=DEV)
    d_out = torch.zeros(n_t, dtype=torch.int32, device=DEV)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    lpk.lpk_select_fraclen(tl, lpk.LPK_VMAX_U64, lpk.LPK_SEL_THETA, d_vm, d_fin, d_cur, d_out, status)
    torch.cuda.synchronize()
    st = ref.new_status()
    want = [ref.select_fraclen_vmax(vm[t], fin[t] + meta[t][1], meta[t][0], cur[t], st) for t in range(n_t)]
    assert d_out.cpu().tolist() == want
    assert int(status.cpu().numpy().view(np.uint32)[0]) == int(st[0])
    tl.destroy()


@pytest.mark.parametrize("sel", [lpk.LPK_SEL_MOMENTUM, lpk.LPK_SEL_SECOND])
def test_reselect_of_the_moment_grids_from_their_maxima(sel):
    """The same rule for the velocity / first moment and the second moment: the maximum is on the state's own grid
    (no comp shift), the width is the state's, the result stays within 15 of the current fraclen; out-of-range
    fraclens are flagged."""
    say("fraclen re-selection of the moments' grids, sel %d" % sel)
    pr = random.Random(50 + sel)
    n_t = 400
    z8 = torch.zeros(16, dtype=torch.int8, device=DEV); z16 = torch.zeros(16, dtype=torch.int16, device=DEV)
    descs, widths = [], []
    for t in range(n_t):
        wm, wu = pr.choice([8, 16]), pr.choice([8, 16])
        descs.append(lpk.make_desc(z8, z8, z16, None, momentum=z8 if wm == 8 else z16, second=z8 if wu == 8 else z16))
        widths.append(wm if sel == lpk.LPK_SEL_MOMENTUM else wu)
    tl = lpk.TensorList(descs)
    mx, fin, cur = [], [], []
    for t in range(n_t):
        W = widths[t]
        mx.append(pr.choice([0, 1, 127, 128, 255, 32767, 32768, (1 << pr.randint(1, 40)) - 1, pr.randint(1, 1 << 38),
                             ((1 << W) - 1) << pr.randint(0, 20), (((1 << W) - 1) << pr.randint(1, 20)) - 1]))
        fi = pr.randint(-64, 64) if pr.random() < .95 else pr.choice([-70, 70])
        fin.append(fi)
        cur.append(max(-64, min(64, fi + pr.randint(-15, 15))) if pr.random() < .97 else 80)
    d_mx = torch.tensor(mx, dtype=torch.int64, device=DEV)
    d_fin = torch.tensor(fin, dtype=torch.int32, device=DEV); d_cur = torch.tensor(cur, dtype=torch.int32, device=DEV)
    d_out = torch.zeros(n_t, dtype=torch.int32, device=DEV)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    lpk.lpk_select_fraclen(tl, lpk.LPK_VMAX_U64, sel, d_mx, d_fin, d_cur, d_out, status)
    torch.cuda.synchronize()
    st = ref.new_status()
    want = [ref.select_fraclen_vmax(mx[t], fin[t], widths[t], cur[t], st) for t in range(n_t)]
    assert d_out.cpu().tolist() == want
    assert int(status.cpu().numpy().view(np.uint32)[0]) == int(st[0])
    tl.destroy()


def test_host_side_argument_errors_with_a_live_list():
    say("argument errors")
    t = torch.zeros(64, dtype=torch.int8, device=DEV)
    g = torch.zeros(64, dtype=torch.int16, device=DEV)
    tl = lpk.TensorList([lpk.make_desc(t, t.clone(), g)])          # no fp32 source
    fl = torch.zeros(1, dtype=torch.int32, device=DEV)
    L = lpk.lib()
    assert L.lpk_kahan_sgd_step(tl.handle, fl.data_ptr(), fl.data_ptr(), fl.data_ptr(), 65536, 0, None, None, None) == lpk.LPK_ERR_INVALID_ARG
    assert L.lpk_kahan_sgd_step(tl.handle, fl.data_ptr(), None, fl.data_ptr(), 1, 0, None, None, None) == lpk.LPK_ERR_INVALID_ARG
    assert L.lpk_quantize_tensor(tl.handle, lpk.LPK_SEL_GRAD, fl.data_ptr(), None, None) == lpk.LPK_ERR_INVALID_ARG
    assert L.lpk_select_fraclen(tl.handle, lpk.LPK_F32, 0, None, None, fl.data_ptr(), fl.data_ptr(), None, None) == lpk.LPK_ERR_INVALID_ARG
    assert L.lpk_select_fraclen(tl.handle, 3, 0, None, None, fl.data_ptr(), fl.data_ptr(), None, None) == lpk.LPK_ERR_INVALID_ARG
    assert L.lpk_select_fraclen(tl.handle, lpk.LPK_VMAX_U64, 0, None, None, fl.data_ptr(), fl.data_ptr(), None, None) == lpk.LPK_ERR_INVALID_ARG
    # the one-pass selection + quantization: no fp32 source, NULL arrays, a destination it does not have
    assert L.lpk_select_quantize(tl.handle, lpk.LPK_SEL_GRAD, fl.data_ptr(), fl.data_ptr(), None, None) == lpk.LPK_ERR_INVALID_ARG
    src = torch.zeros(64, dtype=torch.float32, device=DEV)
    tl2 = lpk.TensorList([lpk.make_desc(t, t.clone(), g, src)])
    assert L.lpk_select_quantize(tl2.handle, lpk.LPK_SEL_GRAD, None, fl.data_ptr(), None, None) == lpk.LPK_ERR_INVALID_ARG
    assert L.lpk_select_quantize(tl2.handle, lpk.LPK_SEL_GRAD, fl.data_ptr(), None, None, None) == lpk.LPK_ERR_INVALID_ARG
    assert L.lpk_select_quantize(tl2.handle, lpk.LPK_SEL_MOMENTUM, fl.data_ptr(), fl.data_ptr(), None, None) == lpk.LPK_ERR_INVALID_ARG
    assert L.lpk_select_quantize(None, lpk.LPK_SEL_GRAD, fl.data_ptr(), fl.data_ptr(), None, None) == lpk.LPK_ERR_INVALID_ARG
    assert L.lpk_select_quantize(tl2.handle, lpk.LPK_SEL_GRAD, fl.data_ptr(), fl.data_ptr(), None, None) == lpk.LPK_OK   # status may be NULL
    torch.cuda.synchronize()
    tl2.destroy()
    assert L.lpk_tensor_list_size(tl.handle) == 1 and L.lpk_tensor_list_tiles(tl.handle) == 1
    # options: unknown code, launch-shape value out of range
    assert L.lpk_tensor_list_set_option(tl.handle, 99, 1) == lpk.LPK_ERR_INVALID_ARG
    assert L.lpk_tensor_list_set_option(tl.handle, lpk.LPK_OPT_STEP_BLOCKS_PER_CU, 65) == lpk.LPK_ERR_INVALID_ARG
    assert L.lpk_tensor_list_set_option(tl.handle, lpk.LPK_OPT_STEP_BLOCKS_PER_CU, -1) == lpk.LPK_ERR_INVALID_ARG
    assert L.lpk_tensor_list_set_option(None, lpk.LPK_OPT_STORE_ALL, 1) == lpk.LPK_ERR_INVALID_ARG
    assert L.lpk_tensor_list_set_option(tl.handle, lpk.LPK_OPT_QUANT_BLOCKS_PER_CU, 64) == lpk.LPK_OK
    tl.destroy()


@pytest.mark.parametrize("mode", ["plain", "momentum", "adam"])
def test_results_do_not_depend_on_the_launch_shape(mode):
    """Every family of kernels under 1, 3, 8 and 64 workgroups per CU (and back to the built-in choice) on a ragged
    multi-tensor set and on a one-tensor workload: whole steps, bit for bit against the oracle."""
    from paper_1810_05486_amd import workloads
    from paper_1810_05486_amd.device_state import DeviceState
    sys.path.insert(0, __file__.rsplit("/", 1)[0])
    from oracle_state import OracleState, draw_grads
    say("launch shapes, %s" % mode)
    opts = (lpk.LPK_OPT_STEP_BLOCKS_PER_CU, lpk.LPK_OPT_DENSE_BLOCKS_PER_CU, lpk.LPK_OPT_ADAM_BLOCKS_PER_CU,
            lpk.LPK_OPT_SCAN_BLOCKS_PER_CU, lpk.LPK_OPT_QUANT_BLOCKS_PER_CU)
    for cfg in (workloads.config(3), workloads.config(5, big_elems=(1 << 21) + 5, n_tiny=3)):
        nt = cfg.n_tensors
        kw = dict(mom_bits=[16] * nt, fl_mom0=24) if mode != "plain" else {}
        if mode == "adam":
            kw.update(sec_bits=[16] * nt, fl_sec0=38)
        dev, host = DeviceState(cfg, **kw), OracleState(cfg, **kw)
        views = dev.host_src_views()
        theta0 = [cfg.theta0(t, out=views[t]).copy() for t in range(nt)]
        dev.upload_src()
        dev.init_theta()
        host.init_theta(theta0)
        for s, per_cu in enumerate((1, 3, 8, 64, 0)):
            for o in opts:
                lpk.lpk_tensor_list_set_option(dev.lists[0], o, per_cu)
            grads = draw_grads(cfg, s, views)
            dev.upload_src()
            if mode == "adam":
                hyper = workloads.adam_hyper(s)
                dev.quantize_grads()
                dev.update_adam(hyper)
                host.update_adam(hyper, grads)
            else:
                mu = 58982 if mode == "momentum" else None
                dev.step(s, mu_q16=mu)
                host.step(s, grads, mu_q16=mu)
            th, co, fl_t, fl_g, vm, status = dev.download()
            ctx = (mode, cfg.id, per_cu)
            assert status == int(host.status[0]) == 0, ctx
            assert fl_g.tolist() == host.fl_grad and vm.tolist() == host.vmax, ctx
            for t in range(nt):
                assert np.array_equal(th[t], host.theta[t]) and np.array_equal(co[t], host.comp[t]), (ctx, t)
                if mode != "plain":
                    assert np.array_equal(dev.mom[t].cpu().numpy(), host.mom[t]), (ctx, t)
                if mode == "adam":
                    assert np.array_equal(dev.sec[t].cpu().numpy(), host.sec[t]), (ctx, t)
        dev.close()


def test_fused_step_with_special_gradient_values():
    """NaN / Inf / subnormal / huge fp32 gradients through the fused call: same theta, comp, vmax and status as
    quantizing first (oracle), for the vector path and for a misaligned tensor."""
    say("fused step, special fp32 values")
    rng = np.random.default_rng(12)
    f = np.float32
    for mis in (0, 1):
        n = 3 * 4096 + 9
        x = (rng.standard_normal(n) * 1e-3).astype(f)
        x[5], x[77], x[4096], x[4097], x[9000], x[n - 1] = np.nan, np.inf, -np.inf, 1e-45, 3e38, -0.0
        theta = rng.integers(-128, 128, size=n).astype(np.int8); comp = rng.integers(-64, 64, size=n).astype(np.int8)
        bt = torch.zeros(n + 64, dtype=torch.int8, device=DEV); dt = bt[mis:mis + n]; dt.copy_(torch.from_numpy(theta))
        bc = torch.zeros(n + 64, dtype=torch.int8, device=DEV); dc = bc[mis:mis + n]; dc.copy_(torch.from_numpy(comp))
        dg = torch.zeros(n, dtype=torch.int16, device=DEV)
        dx = torch.from_numpy(x).to(DEV)
        tl = lpk.TensorList([lpk.make_desc(dt, dc, dg, dx)])
        i32 = dict(dtype=torch.int32, device=DEV)
        for fl_g in (22, -64, 10):
            fl_t, fl_gd = torch.tensor([7], **i32), torch.tensor([fl_g], **i32)
            vmax = torch.zeros(1, dtype=torch.int64, device=DEV); status = torch.zeros(1, dtype=torch.int32, device=DEV)
            lpk.lpk_kahan_sgd_step_f32grad(tl, fl_t, fl_t, fl_gd, 655, 0, vmax, status)
            torch.cuda.synchronize()
            st = ref.new_status()
            g = ref.quantize(x, 16, fl_g, st)
            wv = ref.kahan_sgd_step(theta, comp, g, 7, 7, 7, fl_g, 655, 0, st)
            assert np.array_equal(dt.cpu().numpy(), theta) and np.array_equal(dc.cpu().numpy(), comp), (mis, fl_g)
            assert int(vmax.item()) == wv and int(status.cpu().numpy().view(np.uint32)[0]) == int(st[0]) == ref.STATUS_NONFINITE
        assert int(dg.count_nonzero().item()) == 0
        tl.destroy()


def test_calls_follow_the_stream_they_are_given():
    """Every call takes its hipStream_t explicitly: the whole path enqueued on a side stream (default priority),
    ordered after the upload by an event, while the default stream is kept busy with unrelated work."""
    say("explicit side stream")
    rng = np.random.default_rng(11)
    n = 3 * 4096 + 19
    x = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    theta = rng.integers(-100, 100, size=n).astype(np.int8); comp = rng.integers(-60, 60, size=n).astype(np.int8)
    side = torch.cuda.Stream()
    d_src = torch.from_numpy(x).to(DEV)
    d_theta = torch.from_numpy(theta).to(DEV); d_comp = torch.from_numpy(comp).to(DEV)
    d_grad = torch.zeros(n, dtype=torch.int16, device=DEV)
    fl_t = torch.tensor([7], dtype=torch.int32, device=DEV); fl_g = torch.tensor([15], dtype=torch.int32, device=DEV)
    vmax = torch.zeros(1, dtype=torch.int64, device=DEV); status = torch.zeros(1, dtype=torch.int32, device=DEV)
    tl = lpk.TensorList([lpk.make_desc(d_theta, d_comp, d_grad, d_src)])
    ready = torch.cuda.Event()
    ready.record()                                         # inputs are on the device once the default stream gets here
    busy = torch.zeros(1 << 24, dtype=torch.float32, device=DEV)
    for _ in range(20):
        busy.add_(1.0)                                     # unrelated default-stream work in flight meanwhile
    side.wait_event(ready)
    lpk.lpk_select_fraclen(tl, lpk.LPK_F32, lpk.LPK_SEL_GRAD, None, None, fl_g, fl_g, status, stream=side)
    lpk.lpk_quantize_tensor(tl, lpk.LPK_SEL_GRAD, fl_g, status, stream=side)
    lpk.lpk_kahan_sgd_step(tl, fl_t, fl_t, fl_g, 6554, 0, vmax, status, stream=side)
    side.synchronize()
    torch.cuda.synchronize()
    want_fl = ref.select_fraclen_f32(x, 16, 15)
    g = ref.quantize(x, 16, want_fl)
    want_v = ref.kahan_sgd_step(theta, comp, g, 7, 7, 7, want_fl, 6554)
    assert int(fl_g.item()) == want_fl and int(vmax.item()) == want_v and int(status.item()) == 0
    assert np.array_equal(d_grad.cpu().numpy(), g)
    assert np.array_equal(d_theta.cpu().numpy(), theta) and np.array_equal(d_comp.cpu().numpy(), comp)
    assert float(busy[0].item()) == 20.0
    tl.destroy()


def test_a_list_of_empty_tensors_is_a_no_op():
    """n = 0 for every tensor: no tiles, nothing launched over data; fraclens fall back to their defaults, the
    maxima are cleared, the status word stays clean -- for every entry point."""
    say("all-empty list")
    e8 = torch.zeros(0, dtype=torch.int8, device=DEV); e16 = torch.zeros(0, dtype=torch.int16, device=DEV)
    ef = torch.zeros(0, dtype=torch.float32, device=DEV)
    tl = lpk.TensorList([lpk.make_desc(e8, e8, e16, ef, momentum=e16, second=e16) for _ in range(3)])
    assert tl.n_tiles == 0
    i32 = dict(dtype=torch.int32, device=DEV)
    fl = torch.tensor([3, -4, 60], **i32); fl_bad = torch.tensor([99, 99, 99], **i32)     # out-of-domain values must not matter
    out = torch.full((3,), 77, **i32)
    mx = [torch.full((3,), 9, dtype=torch.int64, device=DEV) for _ in range(3)]
    status = torch.zeros(1, **i32)
    lpk.lpk_select_fraclen(tl, lpk.LPK_F32, lpk.LPK_SEL_GRAD, None, None, fl, out, status)
    lpk.lpk_quantize_tensor(tl, lpk.LPK_SEL_GRAD, fl, status)
    lpk.lpk_quantize_tensor(tl, lpk.LPK_SEL_GRAD, fl_bad, status)
    out2 = torch.full((3,), 77, **i32)
    lpk.lpk_select_quantize(tl, lpk.LPK_SEL_GRAD, fl_bad, out2, status)       # an empty tensor keeps the guess, whatever it is
    torch.cuda.synchronize()
    assert out2.cpu().tolist() == [99, 99, 99]
    lpk.lpk_kahan_sgd_step(tl, fl_bad, fl_bad, fl_bad, 655, 7, mx[0], status)
    lpk.lpk_kahan_sgd_step_f32grad(tl, fl_bad, fl_bad, fl_bad, 655, 0, mx[0], status)
    lpk.lpk_momentum_sgd_step(tl, fl_bad, fl_bad, fl_bad, fl_bad, fl_bad, 655, 58982, 0, mx[0], mx[1], status)
    lpk.lpk_adam_step(tl, fl_bad, fl_bad, fl_bad, fl_bad, fl_bad, fl_bad, fl_bad, (66, 0, 58982, 65470, 0, 0), mx[0], mx[1], mx[2], status)
    torch.cuda.synchronize()
    assert out.cpu().tolist() == [3, -4, 60]
    assert all(m.cpu().tolist() == [0, 0, 0] for m in mx) and int(status.item()) == 0
    tl.destroy()


def test_tensor_longer_than_2_to_the_32_elements():
    """Element offsets past 32 bits: one int8 tensor of 2^32 + 3 tiles + 5 elements, one update straight through the
    C ABI, every byte and vmax compared with the oracle (host threads over contiguous ranges)."""
    say("tensor of 2^32 + 12293 elements")
    n = (1 << 32) + 3 * 4096 + 5
    rng = np.random.default_rng(21)
    blk = 1 << 24

    def tiled(lo, hi, dtype):
        base = rng.integers(lo, hi, size=blk + 1237).astype(dtype)      # period not a power of two
        reps = n // base.size + 1
        return np.tile(base, reps)[:n].copy()
    theta, comp, grad = tiled(-128, 128, np.int8), tiled(-128, 128, np.int8), tiled(-32768, 32768, np.int16)
    d_theta, d_comp, d_grad = (torch.from_numpy(a).to(DEV) for a in (theta, comp, grad))
    tl = lpk.TensorList([lpk.make_desc(d_theta, d_comp, d_grad, None)])
    assert tl.n_tiles == (n + 4095) // 4096
    i32 = dict(dtype=torch.int32, device=DEV)
    fl_t, fl_g = torch.tensor([7], **i32), torch.tensor([14], **i32)
    vmax = torch.zeros(1, dtype=torch.int64, device=DEV); status = torch.zeros(1, **i32)
    lpk.lpk_kahan_sgd_step(tl, fl_t, fl_t, fl_g, 40000, 0, vmax, status)
    torch.cuda.synchronize()
    say("  device step done; oracle on the host ...")
    want_v = ref.kahan_sgd_step_mt(theta, comp, grad, 7, 7, 7, 14, 40000, threads=16)
    assert int(vmax.item()) == want_v and int(status.item()) == 0
    got_t, got_c = d_theta.cpu().numpy(), d_comp.cpu().numpy()
    assert np.array_equal(got_t, theta) and np.array_equal(got_c, comp)
    tl.destroy()


def test_select_and_quantize_longer_than_2_to_the_32_elements():
    """The same length through the max-abs selection and the quantization kernel: the maximum sits past the 2^32-th
    element, so a wrapped offset would lose it."""
    say("select + quantize over 2^32 + 12293 elements")
    n = (1 << 32) + 3 * 4096 + 5
    rng = np.random.default_rng(22)
    base = (rng.standard_normal((1 << 24) + 1237) * 1e-3).astype(np.float32)
    x = np.tile(base, n // base.size + 1)[:n].copy()
    x[n - 7] = 0.0625                                       # the maximum, in the last partial tile
    d_src = torch.from_numpy(x).to(DEV)
    d_theta = torch.zeros(n, dtype=torch.int8, device=DEV); d_grad = torch.zeros(n, dtype=torch.int16, device=DEV)
    tl = lpk.TensorList([lpk.make_desc(d_theta, None, d_grad, d_src)])
    fl = torch.tensor([15], dtype=torch.int32, device=DEV); status = torch.zeros(1, dtype=torch.int32, device=DEV)
    lpk.lpk_select_fraclen(tl, lpk.LPK_F32, lpk.LPK_SEL_GRAD, None, None, fl, fl, status)
    lpk.lpk_quantize_tensor(tl, lpk.LPK_SEL_GRAD, fl, status)
    torch.cuda.synchronize()
    say("  device done; oracle on the host ...")
    want_fl = ref.select_fraclen_f32(x, 16, 15)
    assert want_fl == 18 and int(fl.item()) == want_fl and int(status.item()) == 0      # 0.0625 * 2^18 = 16384 fits, 2^19 does not
    want = ref.quantize_mt(x, 16, want_fl, threads=16)
    assert np.array_equal(d_grad.cpu().numpy(), want)
    # the same through the one-pass call: with the guess that holds, and with one that is wrong (the whole tensor again)
    for guess in (want_fl, want_fl + 1):
        d_grad.zero_()
        fl.fill_(guess)
        lpk.lpk_select_quantize(tl, lpk.LPK_SEL_GRAD, fl, fl, status)
        torch.cuda.synchronize()
        assert int(fl.item()) == want_fl and int(status.item()) == 0, guess
        assert torch.equal(d_grad.cpu(), torch.from_numpy(want)), guess
    tl.destroy()


@pytest.mark.parametrize("store_all", [0, 1])
@pytest.mark.parametrize("tb,cb", [(8, 8), (8, 16), (16, 16)])
def test_lazy_stores_in_every_regime(tb, cb, store_all):
    """Stores of unchanged 16-byte groups are not issued (unless LPK_OPT_STORE_ALL): gradients crafted so that within
    one tensor some wave-sized runs change nothing, some change in one lane, some in a dozen lanes, some everywhere,
    in an order that makes a wave switch between its sparse and dense forms; int16 and fp32 gradient entry points,
    four steps, every byte against the oracle after each."""
    say("lazy stores, theta int%d, comp int%d, store_all=%d" % (tb, cb, store_all))
    rng = np.random.default_rng(40 + tb + cb + store_all)
    n = 70 * 4096 + 1000                                   # 70 full tiles and a ragged one: several per wave of a small grid
    theta = rng.integers(-100, 100, size=n).astype(NP[tb])
    comp = np.zeros(n, dtype=NP[cb])
    d = cb - 1
    fl_t, fl_g = 7, (10 if cb == 8 else 19)                # step shift 12 (13): the 32-bit arithmetic, where stores are lazy
    d_theta = torch.from_numpy(theta).to(DEV); d_comp = torch.from_numpy(comp).to(DEV)
    d_grad = torch.zeros(n, dtype=torch.int16, device=DEV); d_src = torch.zeros(n, dtype=torch.float32, device=DEV)
    tl = lpk.TensorList([lpk.make_desc(d_theta, d_comp, d_grad, d_src)])
    lpk.lpk_tensor_list_set_option(tl, lpk.LPK_OPT_STORE_ALL, store_all)
    i32 = dict(dtype=torch.int32, device=DEV)
    a_fl_t, a_fl_g = torch.tensor([fl_t], **i32), torch.tensor([fl_g], **i32)
    vmax = torch.zeros(1, dtype=torch.int64, device=DEV); status = torch.zeros(1, **i32)
    lr_q = 16384                                           # 1/4: g = 4 moves comp by one theta LSB's worth of 2^(d - 3)
    for step in range(4):
        g = np.zeros(n, dtype=np.int16)
        runs = n // 1024
        kind = rng.integers(0, 5, size=runs)
        kind[(np.arange(runs) // 12) % 2 == 1] = 4                      # stretches where everything changes
        for r in range(runs):
            lo = r * 1024
            if kind[r] == 1:   g[lo + int(rng.integers(0, 1024))] = 8                                   # one lane
            elif kind[r] == 2: g[lo + rng.choice(1024, size=12, replace=False)] = -8                     # about a dozen lanes
            elif kind[r] == 3: g[lo + int(rng.integers(0, 1024))] = 32767                               # theta moves too
            elif kind[r] == 4: g[lo:lo + 1024] = rng.integers(200, 20000, size=1024)                     # everything
        want_v = ref.kahan_sgd_step(theta, comp, g, d, fl_t, fl_t, fl_g, lr_q)
        if step % 2 == 0:
            d_grad.copy_(torch.from_numpy(g))
            lpk.lpk_kahan_sgd_step(tl, a_fl_t, a_fl_t, a_fl_g, lr_q, 0, vmax, status)
        else:                                              # the same integers as exact fp32 values through the fused call
            d_src.copy_(torch.from_numpy(g.astype(np.float32) * np.float32(2.0 ** -fl_g)))
            lpk.lpk_kahan_sgd_step_f32grad(tl, a_fl_t, a_fl_t, a_fl_g, lr_q, 0, vmax, status)
        torch.cuda.synchronize()
        assert int(vmax.item()) == want_v and int(status.item()) == 0, step
        bad_t = int((d_theta.cpu().numpy() != theta).sum()); bad_c = int((d_comp.cpu().numpy() != comp).sum())
        assert bad_t == 0 and bad_c == 0, (step, bad_t, bad_c)
    assert len(np.unique(theta)) > 50 and int(np.abs(comp.astype(np.int64)).max()) > 0
    tl.destroy()


@pytest.mark.parametrize("seed", fuzz_seeds(3))
def test_lazy_stores_random_sparsity(seed):
    """The store-skipping forms of the update on random lists: several tensors of the three vector width pairs, any
    length, gradients that are zero except for random patterns per 1024-element run (nothing, one element, a few,
    one aligned 64-byte stretch of the accumulator, half, everything; small enough to touch only the accumulator
    or large enough to move theta), six steps alternating between the int16 and the fp32 gradient entry points,
    with and without LPK_OPT_STORE_ALL; every byte against the oracle after each step."""
    say("lazy stores: random sparsity, seed %d" % seed)
    rng = np.random.default_rng(3300 + seed)
    pr = random.Random(3400 + seed)
    store_all = seed % 2
    tens = []
    for _ in range(pr.randint(1, 5)):
        tb, cb = pr.choice([(8, 8), (8, 8), (8, 16), (16, 16)])
        n = pr.choice([1000, 4096, 9000, 70 * 4096 + 1000, 33000, 150000])
        t = dict(tb=tb, cb=cb, n=n, d=cb - 1, fl_t=7 if tb == 8 else 12)
        t["fl_g"] = t["fl_t"] + t["d"] - 4                 # step shift 12: the 32-bit arithmetic, where stores are lazy
        t["theta"] = rng.integers(-100, 100, size=n).astype(NP[tb]); t["comp"] = np.zeros(n, dtype=NP[cb])
        t["d_theta"] = torch.from_numpy(t["theta"]).to(DEV); t["d_comp"] = torch.from_numpy(t["comp"]).to(DEV)
        t["d_grad"] = torch.zeros(n, dtype=torch.int16, device=DEV); t["d_src"] = torch.zeros(n, dtype=torch.float32, device=DEV)
        tens.append(t)
    tl = lpk.TensorList([lpk.make_desc(t["d_theta"], t["d_comp"], t["d_grad"], t["d_src"]) for t in tens])
    lpk.lpk_tensor_list_set_option(tl, lpk.LPK_OPT_STORE_ALL, store_all)
    i32 = dict(dtype=torch.int32, device=DEV)
    a_fl_t = torch.tensor([t["fl_t"] for t in tens], **i32); a_fl_g = torch.tensor([t["fl_g"] for t in tens], **i32)
    vmax = torch.zeros(len(tens), dtype=torch.int64, device=DEV); status = torch.zeros(1, **i32)
    lr_q = 16384
    for step in range(6):
        fused = pr.random() < 0.5
        want_v = []
        for t in tens:
            n = t["n"]
            g = np.zeros(n, dtype=np.int16)
            mode = pr.choice(["mixed", "mixed", "none", "all", "rare"])
            for lo in range(0, n, 1024):
                m = min(1024, n - lo)
                k = {"none": 0, "all": 5, "rare": pr.choice([0] * 15 + [1])}.get(mode, pr.randint(0, 5))
                big = pr.random() < 0.2
                val = (lambda size: rng.integers(3000, 30000, size=size) * rng.choice([-1, 1], size=size)) if big else \
                      (lambda size: rng.choice([8, -8, 16, 4, -4], size=size))
                if k == 1:   g[lo + pr.randrange(m)] = val(1)[0]
                elif k == 2: idx = rng.choice(m, size=min(m, pr.randint(2, 20)), replace=False); g[lo + idx] = val(idx.size)
                elif k == 3: a = (pr.randrange(m) // 64) * 64; w = min(64, m - a); g[lo + a:lo + a + w] = val(w)
                elif k == 4: idx = rng.choice(m, size=m // 2, replace=False); g[lo + idx] = val(idx.size)
                elif k == 5: g[lo:lo + m] = val(m)
            want_v.append(ref.kahan_sgd_step(t["theta"], t["comp"], g, t["d"], t["fl_t"], t["fl_t"], t["fl_g"], lr_q))
            if fused:
                t["d_src"].copy_(torch.from_numpy(g.astype(np.float32) * np.float32(2.0 ** -t["fl_g"])))
            else:
                t["d_grad"].copy_(torch.from_numpy(g))
        if fused:
            lpk.lpk_kahan_sgd_step_f32grad(tl, a_fl_t, a_fl_t, a_fl_g, lr_q, 0, vmax, status)
        else:
            lpk.lpk_kahan_sgd_step(tl, a_fl_t, a_fl_t, a_fl_g, lr_q, 0, vmax, status)
        torch.cuda.synchronize()
        assert vmax.cpu().tolist() == want_v and int(status.item()) == 0, (step, fused)
        for i, t in enumerate(tens):
            bad_t = int((t["d_theta"].cpu().numpy() != t["theta"]).sum()); bad_c = int((t["d_comp"].cpu().numpy() != t["comp"]).sum())
            assert bad_t == 0 and bad_c == 0, (step, fused, i, t["tb"], t["cb"], t["n"], bad_t, bad_c)
    tl.destroy()


@pytest.mark.parametrize("store_all", [0, 1])
def test_all_int8_update_with_int8_gradients(store_all):
    """The all-8-bit mode of Section 4 (int8 theta, int8 accumulator, int8 gradients) on the vector path: sparse and
    dense steps, a weight-decay step and a step onto a finer grid (wide arithmetic), several tiles and a ragged tail,
    every byte against the oracle."""
    say("int8 theta + comp + gradients, store_all=%d" % store_all)
    rng = np.random.default_rng(900 + store_all)
    n = 37 * 4096 + 4090
    theta = rng.integers(-100, 100, size=n).astype(np.int8)
    comp = rng.integers(-50, 50, size=n).astype(np.int8)
    d_theta = torch.from_numpy(theta).to(DEV); d_comp = torch.from_numpy(comp).to(DEV)
    d_grad = torch.zeros(n, dtype=torch.int8, device=DEV); d_src = torch.zeros(n, dtype=torch.float32, device=DEV)
    tl = lpk.TensorList([lpk.make_desc(d_theta, d_comp, d_grad, d_src)])
    lpk.lpk_tensor_list_set_option(tl, lpk.LPK_OPT_STORE_ALL, store_all)
    i32 = dict(dtype=torch.int32, device=DEV)
    vmax = torch.zeros(1, dtype=torch.int64, device=DEV); status = torch.zeros(1, **i32)
    #        fl_in fl_out fl_g  lr     wd    gradients
    plan = [(7,    7,     9,    655,   0,    "sparse"),
            (7,    7,     4,    16384, 0,    "dense"),
            (7,    7,     6,    6554,  7,    "dense"),
            (7,    8,     6,    6554,  0,    "dense"),
            (8,    8,     9,    655,   0,    "sparse")]
    for step, (fl_in, fl_out, fl_g, lr_q, wd_q, kind) in enumerate(plan):
        g = rng.integers(-128, 128, size=n).astype(np.int8)
        if kind == "sparse":
            g[rng.random(n) > 0.002] = 0
        want_v = ref.kahan_sgd_step(theta, comp, g, 7, fl_in, fl_out, fl_g, lr_q, wd_q)
        d_grad.copy_(torch.from_numpy(g))
        lpk.lpk_kahan_sgd_step(tl, torch.tensor([fl_in], **i32), torch.tensor([fl_out], **i32), torch.tensor([fl_g], **i32),
                               lr_q, wd_q, vmax, status)
        torch.cuda.synchronize()
        assert int(vmax.item()) == want_v and int(status.item()) == 0, step
        bad_t = int((d_theta.cpu().numpy() != theta).sum()); bad_c = int((d_comp.cpu().numpy() != comp).sum())
        assert bad_t == 0 and bad_c == 0, (step, bad_t, bad_c)
    # the same mode fed from fp32 gradients: quantized to 8 bits in registers (values beyond the int8 rails saturate)
    src = (rng.standard_normal(n) * 0.1).astype(np.float32)
    st = ref.new_status()
    g = ref.quantize(src, 8, 9, st)
    want_v = ref.kahan_sgd_step(theta, comp, g, 7, 8, 8, 9, 6554, 0, st)
    d_src.copy_(torch.from_numpy(src)); d_grad.zero_()
    lpk.lpk_kahan_sgd_step_f32grad(tl, torch.tensor([8], **i32), torch.tensor([8], **i32), torch.tensor([9], **i32), 6554, 0, vmax, status)
    torch.cuda.synchronize()
    assert int(vmax.item()) == want_v and int(status.item()) == int(st[0]) == 0
    assert int(g.min()) == -128 and int(g.max()) == 127 and not d_grad.any().item()
    assert np.array_equal(d_theta.cpu().numpy(), theta) and np.array_equal(d_comp.cpu().numpy(), comp)
    tl.destroy()


@pytest.mark.parametrize("mode", ["plain", "momentum", "adam"])
@pytest.mark.parametrize("n_tensors,p_empty,small_launch", [(1, 0.0, True), (257, 0.05, True), (700, 0.05, False),
                                                            (4096, 0.93, True), (4097, 0.93, False)])
def test_fraclens_and_maxima_on_both_sides_of_the_launch_size_where_the_last_workgroup_finishes_them(n_tensors, p_empty, small_launch, mode):
    """Small launches (at most 128 workgroups, i.e. 512 tiles, over at most 4096 tensors) have their per-tensor results
    (fraclens from the max-abs scan; vmax, mmax, umax of the update kernels) finished by the launch's last workgroup,
    larger ones by separate launches.  Both sides of both limits, and list lengths around multiples of the block
    size, against the oracle tensor by tensor -- twice in a row, the second time with a far smaller gradient and a
    quarter of the state, so a maximum left over from the first call (an accumulator that was not put back to zero)
    would show."""
    say("last-workgroup results: %d tensors, %s" % (n_tensors, mode))
    rng = np.random.default_rng(1000 + n_tensors)
    p = np.array([.1, .2, .2, .2, .15, .05, .05]) * (1 - p_empty) / .95
    sizes = rng.choice([0, 1, 7, 16, 64, 300, 4096, 5000], size=n_tensors, p=[p_empty] + list(p))
    if n_tensors == 1:
        sizes[:] = 5000
    n_tiles = int(((sizes + 4095) // 4096).sum())
    assert (n_tiles <= 512 and n_tensors <= 4096) == small_launch, (n_tiles, n_tensors)
    starts = np.concatenate([[0], np.cumsum((sizes + 15) // 16 * 16)])      # every tensor 16-element aligned
    total = int(starts[-1]) + 16
    theta = rng.integers(-128, 128, total).astype(np.int8)
    comp = rng.integers(-128, 128, total).astype(np.int8)
    mom = rng.integers(-2000, 2000, total).astype(np.int16)
    sec = rng.integers(0, 3000, total).astype(np.int16)
    d_theta, d_comp, d_mom, d_sec = (torch.from_numpy(a.copy()).to(DEV) for a in (theta, comp, mom, sec))
    d_grad = torch.zeros(total, dtype=torch.int16, device=DEV)
    d_src = torch.zeros(total, dtype=torch.float32, device=DEV)
    sl = [slice(int(starts[t]), int(starts[t]) + int(sizes[t])) for t in range(n_tensors)]
    tl = lpk.TensorList([lpk.make_desc(d_theta[s], d_comp[s], d_grad[s], d_src[s], momentum=d_mom[s], second=d_sec[s])
                         for s in sl])
    i32 = dict(dtype=torch.int32, device=DEV)
    fl_t = rng.integers(5, 9, n_tensors); fl_m = rng.integers(12, 16, n_tensors); fl_u = rng.integers(24, 28, n_tensors)
    fl_g0 = rng.integers(10, 14, n_tensors)                                 # defaults: kept by empty and all-zero tensors
    d_fl_t, d_fl_m, d_fl_u, d_fl_g0 = (torch.tensor(a, **i32) for a in (fl_t, fl_m, fl_u, fl_g0))
    hyper = (66, 0, 58982, 65470, 43, 10)
    scale = 2.0 ** rng.integers(-12, -3, n_tensors)
    for rnd in range(2):
        src = rng.standard_normal(total).astype(np.float32)
        for t in range(n_tensors):
            src[sl[t]] *= scale[t] * (1.0 if rnd == 0 else 1.0 / 256)
        src[sl[n_tensors // 2]] = 0.0                                        # an all-zero tensor keeps its default
        d_src.copy_(torch.from_numpy(src))
        d_fl_g = torch.full((n_tensors,), -77, **i32)
        mx = [torch.full((n_tensors,), 99, dtype=torch.int64, device=DEV) for _ in range(3)]
        status = torch.zeros(1, **i32)
        lpk.lpk_select_fraclen(tl, lpk.LPK_F32, lpk.LPK_SEL_GRAD, None, None, d_fl_g0, d_fl_g, status)
        lpk.lpk_quantize_tensor(tl, lpk.LPK_SEL_GRAD, d_fl_g, status)
        if mode == "plain":
            lpk.lpk_kahan_sgd_step(tl, d_fl_t, d_fl_t, d_fl_g, 6554, 0, mx[0], status)
        elif mode == "momentum":
            lpk.lpk_momentum_sgd_step(tl, d_fl_t, d_fl_t, d_fl_m, d_fl_m, d_fl_g, 6554, 58982, 0, mx[0], mx[1], status)
        else:
            lpk.lpk_adam_step(tl, d_fl_t, d_fl_t, d_fl_m, d_fl_m, d_fl_u, d_fl_u, d_fl_g, hyper, mx[0], mx[1], mx[2], status)
        torch.cuda.synchronize()
        st = ref.new_status()
        want_fl, want_mx = [], [[], [], []]
        for t in range(n_tensors):
            s = sl[t]
            fl = ref.select_fraclen_f32(src[s], 16, int(fl_g0[t]), st)
            g = ref.quantize(src[s], 16, fl, st)
            if mode == "plain":
                m = (ref.kahan_sgd_step(theta[s], comp[s], g, 7, fl_t[t], fl_t[t], fl, 6554, 0, st), 0, 0)
            elif mode == "momentum":
                m = ref.momentum_sgd_step(theta[s], comp[s], mom[s], g, 7, fl_t[t], fl_t[t], fl_m[t], fl_m[t], fl, 6554, 58982, 0, st) + (0,)
            else:
                m = ref.adam_step(theta[s], comp[s], mom[s], sec[s], g, 7, fl_t[t], fl_t[t], fl_m[t], fl_m[t], fl_u[t], fl_u[t], fl, *hyper, st)
            want_fl.append(fl)
            for k in range(3):
                want_mx[k].append(m[k])
        ctx = (n_tensors, mode, rnd)
        assert d_fl_g.cpu().tolist() == want_fl, ctx
        n_max = {"plain": 1, "momentum": 2, "adam": 3}[mode]
        for k in range(n_max):
            assert mx[k].cpu().tolist() == want_mx[k], ctx + (k,)
        for k in range(n_max, 3):
            assert mx[k].cpu().tolist() == [99] * n_tensors, ctx + (k,)      # arrays the call was not given stay untouched
        assert np.array_equal(d_theta.cpu().numpy(), theta) and np.array_equal(d_comp.cpu().numpy(), comp), ctx
        assert np.array_equal(d_mom.cpu().numpy(), mom) and np.array_equal(d_sec.cpu().numpy(), sec), ctx
        assert int(status.cpu().numpy().view(np.uint32)[0]) == int(st[0]), ctx
        for host, dev in ((theta, d_theta), (comp, d_comp), (mom, d_mom), (sec, d_sec)):
            host //= 4
            dev.copy_(torch.from_numpy(host))
    tl.destroy()


@pytest.mark.parametrize("seed", fuzz_seeds(3))
def test_select_and_quantize_random_lists(seed):
    """Max-abs fraclen selection followed by quantization on random lists: any size, sources that are only 4-byte
    aligned, 8- and 16-bit destinations (the gradient array or theta), magnitudes anywhere in fp32's range, the
    tensor's maximum planted on both sides of the significand edge of the fraclen rule, and now and then zeros only,
    subnormals only, a NaN or an infinity."""
    say("select + quantize: random lists, seed %d" % seed)
    rng = np.random.default_rng(3100 + seed)
    pr = random.Random(3200 + seed)
    f = np.float32
    for rep in range(4):
        sel = pr.choice([lpk.LPK_SEL_GRAD, lpk.LPK_SEL_THETA])
        xs, bits, keep, descs, outs = [], [], [], [], []
        for _ in range(pr.randint(1, 14)):
            n = pr.choice(SIZES + [70001])
            W = pr.choice([8, 16])
            kind = pr.random()
            e = pr.randint(-120, 120)
            if kind < 0.08:
                x = np.zeros(n, dtype=f)
            elif kind < 0.14:
                x = (rng.integers(-200, 200, n).astype(np.int32).view(np.uint32) & np.uint32(0x807fffff)).view(f).copy()   # subnormals
            else:
                with np.errstate(over="ignore"):
                    x = (rng.standard_normal(n) * 2.0 ** e).astype(f)
                if n and kind < 0.6:           # plant a maximum whose significand sits at the edge where the candidate is one too fine
                    E = int(np.clip(127 + e + 3, 1, 254))
                    m = pr.choice([0x7FFFFF, 0x7FFFFF - (1 << (24 - W)) + 1, 0x7FFFFF - (1 << (24 - W)), 0x7FFFFF - (1 << (24 - W)) + 2, 0])
                    x[pr.randrange(n)] = np.array([(E << 23) | m | (pr.getrandbits(1) << 31)], dtype=np.uint32).view(f)[0]
                if n and kind > 0.93:
                    x[pr.randrange(n)] = pr.choice([np.nan, np.inf, -np.inf])
            mis = pr.choice([0, 0, 1, 3, 4])
            sbuf = torch.zeros(n + 16, dtype=torch.float32, device=DEV)
            src = sbuf[mis:mis + n]; src.copy_(torch.from_numpy(x))
            obuf = torch.full((n + 32,), 9, dtype=TT[W], device=DEV)
            omis = pr.choice([0, 0, 1, 8])
            out = obuf[omis:omis + n]
            other = torch.zeros(max(n, 1), dtype=torch.int16 if sel == lpk.LPK_SEL_THETA else torch.int8, device=DEV)[:n]
            descs.append(lpk.make_desc(out, None, other, src) if sel == lpk.LPK_SEL_THETA else lpk.make_desc(other, None, out, src))
            xs.append(x); bits.append(W); keep += [sbuf, obuf, other]; outs.append((obuf, out, omis, n))
        tl = lpk.TensorList(descs)
        lpk.lpk_tensor_list_set_option(tl, lpk.LPK_OPT_QUANT_BLOCKS_PER_CU, pr.choice([0, 0, 1, 3, 8, 64]))   # any launch shape
        lpk.lpk_tensor_list_set_option(tl, lpk.LPK_OPT_SCAN_BLOCKS_PER_CU, pr.choice([0, 0, 1, 3, 8, 64]))
        defaults = [pr.randint(-64, 64) for _ in xs]
        fl = torch.tensor(defaults, dtype=torch.int32, device=DEV)
        fl_out = torch.full((len(xs),), -99, dtype=torch.int32, device=DEV)
        status = torch.zeros(1, dtype=torch.int32, device=DEV)
        lpk.lpk_select_fraclen(tl, lpk.LPK_F32, sel, None, None, fl, fl_out, status)
        lpk.lpk_quantize_tensor(tl, sel, fl_out, status)
        torch.cuda.synchronize()
        st = ref.new_status()
        got_fl = fl_out.cpu().tolist()
        for t, x in enumerate(xs):
            want_fl = ref.select_fraclen_f32(x, bits[t], defaults[t], st)
            assert got_fl[t] == want_fl, (t, x.size, bits[t], got_fl[t], want_fl)
            want_q = ref.quantize(x, bits[t], want_fl, st)
            obuf, out, omis, n = outs[t]
            assert np.array_equal(out.cpu().numpy(), want_q), (t, x.size, bits[t], want_fl)
            host = obuf.cpu().numpy()
            assert (host[:omis] == 9).all() and (host[omis + n:] == 9).all(), ("bytes around the destination written", t)
        assert int(status.cpu().numpy().view(np.uint32)[0]) == int(st[0])
        # the same through lpk_select_quantize, with guesses that hold, miss by one, miss by far, or lie outside the domain
        want_fls = [ref.select_fraclen_f32(x, bits[t], defaults[t]) for t, x in enumerate(xs)]
        for rnd in range(3):
            guesses = []
            for t, x in enumerate(xs):
                zero = x.size == 0 or not np.any(x.view(np.uint32) & np.uint32(0x7fffffff))
                if zero:                       # the guess doubles as the default an empty or all-zero tensor keeps
                    guesses.append(pr.choice([defaults[t], defaults[t], 70, -70]))
                else:
                    guesses.append(pr.choice([want_fls[t], want_fls[t], want_fls[t] + 1, want_fls[t] - 1, pr.randint(-64, 64), 99, -99]))
            for obuf, out, omis, n in outs:
                obuf.fill_(9)
            fl_g = torch.tensor(guesses, dtype=torch.int32, device=DEV)
            inplace = rnd == 2
            fl_o = fl_g if inplace else torch.full((len(xs),), -99, dtype=torch.int32, device=DEV)
            status.zero_()
            lpk.lpk_select_quantize(tl, sel, fl_g, fl_o, status)
            torch.cuda.synchronize()
            st = ref.new_status()
            got_fl = fl_o.cpu().tolist()
            for t, x in enumerate(xs):
                want_fl = ref.select_fraclen_f32(x, bits[t], guesses[t], st)
                assert got_fl[t] == want_fl, ("one pass", rnd, t, x.size, bits[t], guesses[t], got_fl[t], want_fl)
                obuf, out, omis, n = outs[t]
                want_q = np.full(n, 9, dtype=NP[bits[t]])
                ref.quantize(x, bits[t], want_fl, st, out=want_q)            # out of range: flagged, destination untouched
                assert np.array_equal(out.cpu().numpy(), want_q), ("one pass", rnd, t, x.size, bits[t], guesses[t], want_fl)
                host = obuf.cpu().numpy()
                assert (host[:omis] == 9).all() and (host[omis + n:] == 9).all(), ("bytes around the destination written", t)
            assert int(status.cpu().numpy().view(np.uint32)[0]) == int(st[0]), ("one pass", rnd, guesses)
        tl.destroy()

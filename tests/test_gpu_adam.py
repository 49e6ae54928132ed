"""ADAM with the lazy update inside: GPU library vs CPU oracle, bit for bit (needs an MI355X)."""
import random
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

from oracle import ref
from paper_1810_05486_amd import binding as lpk
from paper_1810_05486_amd import workloads
from oracle_state import OracleState, draw_grads

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


def u64(t):
    return t.cpu().numpy().view(np.uint64).tolist()


def compare(dev, host, what):
    th, co, fl_t, fl_g, vm, status = dev.download()
    assert status == int(host.status[0]), (what, "status", status, int(host.status[0]))
    assert fl_t.tolist() == list(host.fl_theta) and fl_g.tolist() == list(host.fl_grad), (what, "fraclens")
    assert dev.fl_mom.cpu().tolist() == list(host.fl_mom), (what, "fl_mom")
    assert dev.fl_sec.cpu().tolist() == list(host.fl_sec), (what, "fl_sec", dev.fl_sec.cpu().tolist()[:8], host.fl_sec[:8])
    assert vm.tolist() == list(host.vmax), (what, "vmax")
    assert u64(dev.mmax) == list(host.mmax), (what, "mmax")
    assert u64(dev.umax) == list(host.umax), (what, "umax")
    for t in range(host.cfg.n_tensors):
        assert np.array_equal(th[t], host.theta[t]), (what, "theta", t)
        assert np.array_equal(co[t], host.comp[t]), (what, "comp", t)
        assert np.array_equal(dev.mom[t].cpu().numpy(), host.mom[t]), (what, "mom", t)
        assert np.array_equal(dev.sec[t].cpu().numpy(), host.sec[t]), (what, "sec", t)


def run_config(cfg, steps, lr=1e-3, eps=1e-8, comp_bits=None, fl_mom0=24, fl_sec0=38, state_bits=16, fused=False):
    from paper_1810_05486_amd.device_state import DeviceState
    bits = [state_bits] * cfg.n_tensors
    kw = dict(comp_bits=comp_bits, mom_bits=bits, sec_bits=bits, fl_mom0=fl_mom0, fl_sec0=fl_sec0)
    dev, host = DeviceState(cfg, **kw), OracleState(cfg, **kw)
    views = dev.host_src_views()
    theta0 = [cfg.theta0(t, out=views[t]).copy() for t in range(cfg.n_tensors)]
    dev.upload_src()
    dev.init_theta()
    host.init_theta(theta0)
    for s in steps:
        grads = draw_grads(cfg, s, views)
        dev.upload_src()
        hyper = workloads.adam_hyper(s, lr=lr, eps=eps)
        if fused:                                          # fp32 gradients straight into the update, no int16 round trip
            dev.select_grads()
            dev.update_adam(hyper, fused=True)
        else:
            dev.quantize_grads()
            dev.update_adam(hyper)
        host.update_adam(hyper, grads)
        compare(dev, host, "config %d step %d" % (cfg.id, s))
    dev.close()
    return host


def test_adam_config1_int8_theta_int16_moments():
    say("adam: config 1, int8 theta and accumulator, int16 moments, 60 steps")
    host = run_config(workloads.config(1), range(60))
    assert int(host.status[0]) == 0
    assert np.abs(host.mom[0].astype(int)).max() > 2000 and host.sec[0].max() > 2000      # both grids settled and in use
    assert len(np.unique(host.theta[0])) > 50


def test_adam_lenet_int16_everything_reselect():
    say("adam: LeNet shapes, all int16, theta and both moment grids re-selected every step")
    run_config(workloads.config(2), range(30), lr=2e-3, eps=1e-6)


def test_adam_resnet50_mixed_widths():
    say("adam: ResNet-50 shapes, int8 theta with the int16 classifier")
    run_config(workloads.config(4), range(4), fl_mom0=36, fl_sec0=60)


def test_adam_int8_theta_with_int16_accumulator():
    say("adam: ResNet-18 shapes, int8 theta with an int16 accumulator (22-bit parameter)")
    cfg = workloads.config(3)
    run_config(cfg, [0, 1, 2, 40], comp_bits=[16] * cfg.n_tensors, fl_mom0=28, fl_sec0=46)


def test_adam_config5_reduced_and_int8_moments():
    say("adam: config 5 shape at reduced size; then 8-bit moments (element path)")
    cfg = workloads.config(5, big_elems=(1 << 22) + 21, n_tiny=200)
    run_config(cfg, range(4))
    run_config(workloads.config(5, big_elems=70001, n_tiny=20), range(3), state_bits=8, fl_mom0=16, fl_sec0=30)


@pytest.mark.parametrize("fused", [False, True])
def test_adam_config5_full_size_in_bench_launch_configuration(fused):
    """The 1 Gi + 10000 x 256 workload at full size, the lists and launch shape `bench.py --adam` times (its
    int16-gradient step, then its fp32-gradient step), every output byte of two steps compared with the oracle (run
    on the host's threads)."""
    say("adam: config 5 at FULL size, 2 steps, fp32 gradients=%s" % fused)
    run_config(workloads.config(5), range(2), fused=fused)


def make_case(rng, n, tb, cb, mb, ub, gb, d, fls, mis=0, sec_lo=0, sec_hi=None, gmax=None, extremes=False):
    """One tensor of a hand-made list: random theta / comp / moments / gradients of the given widths on the host and in
    device buffers shifted by `mis` elements.  fls = (fl_in, fl_out, fl_m_in, fl_m_out, fl_u_in, fl_u_out, fl_g)."""
    c = dict(n=n, tb=tb, cb=cb, mb=mb, ub=ub, gb=gb, d=d, fls=list(fls))
    c["theta"] = rng.integers(-(2 ** (tb - 1)), 2 ** (tb - 1), size=n).astype(NP[tb])
    c["comp"] = rng.integers(-(2 ** (cb - 1)), 2 ** (cb - 1), size=n).astype(NP[cb]) if cb else None
    c["mom"] = rng.integers(-(2 ** (mb - 1)), 2 ** (mb - 1), size=n).astype(NP[mb])
    c["sec"] = rng.integers(sec_lo, sec_hi if sec_hi is not None else 2 ** (ub - 1), size=n).astype(NP[ub])
    glim = gmax if gmax is not None else 2 ** (gb - 1)
    c["grad"] = rng.integers(-glim, glim, size=n).astype(NP[gb])
    if extremes and n >= 16:                       # rails of every operand against each other
        lo_m, hi_m, lo_g, hi_g = -(2 ** (mb - 1)), 2 ** (mb - 1) - 1, -(2 ** (gb - 1)), 2 ** (gb - 1) - 1
        c["mom"][:8] = [hi_m, hi_m, lo_m, lo_m, 0, 0, 1, -1]
        c["grad"][:8] = [hi_g, lo_g, hi_g, lo_g, hi_g, lo_g, 0, 0]
        c["sec"][:8] = [0, 2 ** (ub - 1) - 1, 0, 2 ** (ub - 1) - 1, 1, 2, 3, 0]
        c["sec"][8:16] = [0, 1, 2, 3, 4, 15, 16, 17]
        c["grad"][8:16] = 0

    def dev(a, bits):
        buf = torch.zeros(n + 64, dtype=TT[bits], device=DEV)
        v = buf[mis:mis + n]
        v.copy_(torch.from_numpy(a))
        return buf, v
    c["bufs"] = []
    for key, bits in (("theta", tb), ("comp", cb), ("mom", mb), ("sec", ub), ("grad", gb)):
        if c[key] is None:
            c["d_" + key] = None
            continue
        b, v = dev(c[key], bits)
        c["bufs"].append(b); c["d_" + key] = v
    return c


def run_list(cases, hyper):
    """One lpk_adam_step over the list, the oracle tensor by tensor on the host copies, everything compared."""
    tl = lpk.TensorList([lpk.make_desc(c["d_theta"], c["d_comp"], c["d_grad"], None,
                                       c["d"] if c["cb"] and c["d"] is not None else lpk.LPK_COMP_SHIFT_DEFAULT,
                                       momentum=c["d_mom"], second=c["d_sec"]) for c in cases])
    i32 = dict(dtype=torch.int32, device=DEV)
    arr = [torch.tensor([c["fls"][j] for c in cases], **i32) for j in range(7)]
    vmax, mmax, umax = (torch.full((len(cases),), 5 + k, dtype=torch.int64, device=DEV) for k in range(3))
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    lpk.lpk_adam_step(tl, arr[0], arr[1], arr[2], arr[3], arr[4], arr[5], arr[6], hyper, vmax, mmax, umax, status)
    torch.cuda.synchronize()
    st = ref.new_status()
    for i, c in enumerate(cases):
        dd = c["d"] if c["d"] is not None else (c["cb"] - 1 if c["cb"] else 0)
        f = c["fls"]
        want = ref.adam_step(c["theta"], c["comp"], c["mom"], c["sec"], c["grad"], dd, f[0], f[1], f[2], f[3], f[4], f[5], f[6],
                             *hyper, status=st)
        ctx = {k: c[k] for k in ("n", "tb", "cb", "mb", "ub", "gb", "d", "fls")}
        ctx.update(hyper=hyper, i=i)
        assert np.array_equal(c["d_theta"].cpu().numpy(), c["theta"]), ("theta", ctx)
        if c["cb"]:
            assert np.array_equal(c["d_comp"].cpu().numpy(), c["comp"]), ("comp", ctx)
        assert np.array_equal(c["d_mom"].cpu().numpy(), c["mom"]), ("mom", ctx)
        assert np.array_equal(c["d_sec"].cpu().numpy(), c["sec"]), ("sec", ctx)
        got = (int(vmax[i].item()), int(mmax[i].item()), int(umax[i].item()))
        assert got == want, ("max", got, want, ctx)
    assert int(status.cpu().numpy().view(np.uint32)[0]) == int(st[0])
    tl.destroy()
    return int(st[0])


@pytest.mark.parametrize("seed", fuzz_seeds(4))
def test_adam_random_lists(seed):
    """Random widths, shifts, grid moves, alignments, sizes and hyper-parameters straight through the C ABI,
    including tensors that fall outside the domain (skipped and flagged on both sides)."""
    say("adam: random lists, seed %d" % seed)
    rng = np.random.default_rng(800 + seed)
    pr = random.Random(900 + seed)
    sizes = [0, 1, 15, 16, 17, 255, 1024, 4095, 4096, 4097, 9001, 33000]
    for rep in range(8):
        cases = []
        for _ in range(pr.randint(1, 10)):
            tb = pr.choice([8, 16])
            mb, ub = pr.choice([(16, 16), (16, 16), (16, 16), (8, 16), (16, 8), (8, 8)])
            cb = pr.choice([tb, tb, tb, 8, 16, 0])
            gb = pr.choice([16, 16, 16, 8])
            d = pr.choice([None, None, pr.randint(0, 24)]) if cb else None
            fl_in = pr.randint(-10, 20)
            delta = pr.choice([0, 0, 0, 0, 1, -1, pr.randint(-15, 15)])
            fl_g = pr.randint(0, 40)
            fl_m_in = fl_g + pr.choice([0, 1, -1, pr.randint(-12, 12)])
            fl_m_out = fl_m_in + pr.choice([0, 0, 0, 0, 1, -1, pr.randint(-15, 15)])
            fl_u_in = 2 * fl_g + pr.choice([0, -3, pr.randint(-25, 8), pr.randint(-40, 30)])
            fl_u_out = fl_u_in + pr.choice([0, 0, 0, 0, 1, -1, pr.randint(-15, 15)])
            fls = [max(-64, min(64, f)) for f in (fl_in, fl_in + delta, fl_m_in, fl_m_out, fl_u_in, fl_u_out, fl_g)]
            lo_u = pr.choice([0, 0, 0, -(2 ** (ub - 1))])                       # mostly valid (non-negative) second moments
            cases.append(make_case(rng, pr.choice(sizes), tb, cb, mb, ub, gb, d, fls, mis=pr.choice([0, 0, 0, 1, 8, 16]),
                                   sec_lo=lo_u, sec_hi=pr.choice([4, 300, 2 ** (ub - 1)])))
        hyper = (pr.choice([1, 66, 21000, 65535]), pr.choice([0, 0, 4, 11, pr.randint(0, 48)]),
                 pr.choice([58982, 32768, 0, 65535]), pr.choice([65470, 58982, 0, 65535]),
                 pr.choice([0, 43980, 65535, 1]), pr.choice([0, 26, 10, pr.randint(0, 48)]))
        run_list(cases, hyper)


@pytest.mark.parametrize("seed", fuzz_seeds(3))
def test_adam_standing_grids_around_every_condition_of_the_short_route(seed):
    """The usual case of a running optimizer -- 16-bit moments on grids that stand still, an int8 theta, a small step --
    takes a shorter arithmetic route inside the kernel (fp32 FMA roundings for the first moment and the root, integer
    rounding for the second moment, a reciprocal without refinement).  Lists of aligned tensors whose fraclens and
    hyper-parameters sit on both sides of each condition of that route (first-moment grid 0..8 bits finer than the
    gradient's, or coarser, or further; (1 - beta2) g^2 below / above 2^30 on the second moment's guard grid; step bound
    below / above 2^22; accumulator 8 or 16 bits wide; theta 16 bits wide), operands on their rails, ragged sizes."""
    say("adam: standing grids around the short route's conditions, seed %d" % seed)
    rng = np.random.default_rng(1300 + seed)
    pr = random.Random(1400 + seed)
    for rep in range(10):
        b1 = pr.choice([58982, 58982, 32768, 65535, 1, 62259])
        b2 = pr.choice([65470, 65470, 64881, 65535, 58982])
        lr_q, lr_exp = pr.choice([(33554, 9), (65535, 9), (40000, 4), (33554, 14), (21000, 7), (65535, 2)])
        eps_q, eps_exp = pr.choice([(43980, 26), (0, 0), (65535, 0), (1, 48), (40000, 12)])
        hyper = (lr_q, lr_exp, b1, b2, eps_q, eps_exp)
        cases = []
        for _ in range(pr.randint(3, 9)):
            tb, cb = pr.choice([(8, 8), (8, 8), (8, 8), (8, 16), (16, 16)])
            fl_g = pr.randint(8, 30)
            sh = pr.choice([0, 0, 1, 2, 3, 8, 8, 9, -1, 5])
            fl_m = fl_g + sh
            sh2 = pr.choice([-6, -7, -7, -8, -11, -11, -15, -20, -3])
            fl_u = 2 * fl_g + sh2
            fl_t = pr.choice([7, 7, 5, 10]) if tb == 8 else pr.choice([15, 12])
            if not all(-64 <= f <= 64 for f in (fl_t, fl_m, fl_u, fl_g)):
                continue
            gmax = pr.choice([None, None, 3000, 40])
            cases.append(make_case(rng, pr.choice([16, 4096, 4097, 8200, 33000, 70001]), tb, cb, 16, 16, 16, None,
                                   (fl_t, fl_t, fl_m, fl_m, fl_u, fl_u, fl_g), sec_hi=pr.choice([None, 300, 4]), gmax=gmax,
                                   extremes=True))
        if cases:
            run_list(cases, hyper)


@pytest.mark.parametrize("b2", [0, 1, 58982, 65470, 65535])
def test_adam_short_route_with_negative_second_moments(b2):
    """A negative second moment is a state the optimizer never reaches, but every int16 input has a defined result
    (the new moment is clamped to [0, qmax]).  On the short route the 32-bit sum t4 - (1 - beta2) u passes 2^31 for
    negative u, so both signs are run on standing grids with every beta2 that stretches it (0: the whole of -65536 u),
    the rails of u against the rails of g included, through the 1024-element rows and the groups of 8."""
    say("adam: short route, second moments of both signs, beta2 = %d" % b2)
    rng = np.random.default_rng(1700 + b2)
    hyper = (33554, 9, 58982, b2, 43980, 26)
    cases = []
    for n, tb, cb, sh2 in ((4096 + 1024 + 24, 8, 8, -7), (2048, 8, 8, -11), (8200, 8, 16, -7), (70001, 8, 8, -20)):
        fl_g = 20
        c = make_case(rng, n, tb, cb, 16, 16, 16, None, (7, 7, fl_g + 1, fl_g + 1, 2 * fl_g + sh2, 2 * fl_g + sh2, fl_g),
                      sec_lo=-32768, sec_hi=32768)
        c["sec"][:6] = [-32768, -32768, -32768, -1, -1, 32767]
        c["grad"][:6] = [-32768, 32767, 0, -32768, 0, -32768]
        c["d_sec"].copy_(torch.from_numpy(c["sec"])); c["d_grad"].copy_(torch.from_numpy(c["grad"]))
        cases.append(c)
    run_list(cases, hyper)


def test_adam_argument_errors():
    say("adam: host-side argument errors")
    n = 64
    th = torch.zeros(n, dtype=torch.int8, device=DEV); co = torch.zeros(n, dtype=torch.int8, device=DEV)
    g = torch.zeros(n, dtype=torch.int16, device=DEV); m = torch.zeros(n, dtype=torch.int16, device=DEV)
    u = torch.zeros(n, dtype=torch.int16, device=DEV)
    fl = torch.zeros(1, dtype=torch.int32, device=DEV)
    good = (66, 0, 58982, 65470, 0, 0)
    full = lpk.TensorList([lpk.make_desc(th, co, g, None, momentum=m, second=u)])
    for bad in ((65536, 0, 1, 1, 0, 0), (1, 49, 1, 1, 0, 0), (1, 0, 65536, 1, 0, 0), (1, 0, 1, 1, 65536, 0), (1, 0, 1, 1, 0, 49)):
        with pytest.raises(lpk.LpkError):
            lpk.lpk_adam_step(full, fl, fl, fl, fl, fl, fl, fl, bad)
    with pytest.raises(lpk.LpkError):
        lpk.lpk_adam_step(full, fl, fl, fl, None, fl, fl, fl, good)
    no_second = lpk.TensorList([lpk.make_desc(th, co, g, None, momentum=m)])
    with pytest.raises(lpk.LpkError):
        lpk.lpk_adam_step(no_second, fl, fl, fl, fl, fl, fl, fl, good)
    with pytest.raises(lpk.LpkError):
        lpk.lpk_select_fraclen(no_second, lpk.LPK_VMAX_U64, lpk.LPK_SEL_SECOND, fl, fl, fl, fl)
    lpk.lpk_adam_step(full, fl, fl, fl, fl, fl, fl, fl, good)       # the good call goes through
    torch.cuda.synchronize()
    full.destroy(); no_second.destroy()


def test_adam_fused_fp32_gradient_step_equals_quantize_then_step():
    """lpk_adam_step_f32grad against the oracle's quantize + ADAM step, on every kind of workload."""
    say("fused adam: config 1")
    run_config(workloads.config(1), range(30), fused=True)
    say("fused adam: config 2 (int16 everything, grid moves)")
    run_config(workloads.config(2), range(20), lr=2e-3, eps=1e-6, fused=True)
    say("fused adam: config 4 (mixed widths)")
    run_config(workloads.config(4), range(3), fl_mom0=36, fl_sec0=60, fused=True)
    say("fused adam: config 5 reduced, ragged sizes; int8 theta with an int16 accumulator; 8-bit moments (element path)")
    cfg = workloads.config(5, big_elems=(1 << 22) + 21, n_tiny=200)
    run_config(cfg, range(4), fused=True)
    run_config(cfg, range(3), comp_bits=[16] * cfg.n_tensors, fused=True)
    run_config(workloads.config(5, big_elems=70001, n_tiny=20), range(3), state_bits=8, fl_mom0=16, fl_sec0=30, fused=True)


def random_workload(pr, cid):
    """A small random parameter set with its own training recipe: 1-12 tensors of any rank and length up to 50 000,
    8- or 16-bit parameters per tensor, a learning-rate drop halfway, any of the gradient distributions."""
    shapes = []
    for _ in range(pr.randint(1, 12)):
        r = pr.random()
        if r < 0.3:
            shapes.append((pr.choice([1, 7, 64, 256, 1000, 4096, 4097, 20000]),))
        elif r < 0.8:
            shapes.append((pr.randint(1, 200), pr.randint(1, 250)))
        else:
            shapes.append((pr.randint(1, 24), pr.randint(1, 24), 3, 3))
    bits = [pr.choice([8, 8, 16]) for _ in shapes]
    lr0 = pr.choice([66, 655, 3277, 6554, 32768])
    return workloads.Config(cid, "random workload", shapes, bits, 40, [(0, lr0), (pr.randint(8, 25), max(1, lr0 // pr.choice([2, 10])))],
                            pr.choice([0, 0, 7, 300]), pr.choice(["normal_1e-3", "normal_loguniform", "laplace_1e-4", "normal_fanin"]),
                            pr.random() < 0.5)


@pytest.mark.parametrize("seed", fuzz_seeds(3))
def test_adam_random_workloads_follow_the_oracle_step_by_step(seed):
    """Random parameter sets through 30 consecutive ADAM steps (bias-corrected step size per step, both moment grids
    re-selected every step with the one-step lag: the kernel's short and general arithmetic routes alternate as the
    grids settle), plain or fed from the fp32 gradients; everything after every step."""
    pr = random.Random(4500 + seed)
    cfg = random_workload(pr, 300 + seed)
    fused = pr.random() < 0.4
    say("adam: random workload %d: %d tensors, %d parameters, reselect=%s, fused=%s" % (seed, cfg.n_tensors, cfg.n_params,
                                                                                       cfg.reselect, fused))
    run_config(cfg, range(30), lr=pr.choice([1e-3, 1e-2, 1e-4]), state_bits=pr.choice([16, 16, 8]), fused=fused)


def test_momentum_and_adam_on_a_tensor_longer_than_2_to_the_32_elements():
    """Element offsets past 32 bits in the two optimizer kernels (rows of 1024 and groups of 8 in ADAM, the momentum
    kernel's vector path): one tensor of 2^32 + 3 tiles + 77 elements, filled on the device; elements are independent,
    so the oracle runs on windows -- the start, both sides of the 2^32 boundary, the ragged end, and a few tiles
    picked at random -- downloaded before the step and compared after it."""
    n = (1 << 32) + 3 * 4096 + 77
    say("momentum and ADAM on a tensor of %d elements" % n)
    g = torch.Generator(device=DEV).manual_seed(5)

    def fill(lo, hi, dtype):
        out = torch.empty(n, dtype=dtype, device=DEV)
        step = 1 << 28
        for a in range(0, n, step):                    # in pieces: randint's int64 intermediate stays small
            m = min(step, n - a)
            out[a:a + m] = torch.randint(lo, hi, (m,), generator=g, device=DEV, dtype=torch.int32).to(dtype)
        return out
    d = dict(theta=fill(-128, 128, torch.int8), comp=fill(-128, 128, torch.int8), mom=fill(-3000, 3000, torch.int16),
             sec=fill(0, 3000, torch.int16), grad=fill(-32768, 32768, torch.int16))
    rnd = random.Random(9)
    windows = [(0, 8192), ((1 << 32) - 8192, (1 << 32) + 8192), (n - 5000, n)] + \
              [(t * 4096, t * 4096 + 4096) for t in (rnd.randrange(n // 4096) for _ in range(6))]
    tl = lpk.TensorList([lpk.make_desc(d["theta"], d["comp"], d["grad"], None, momentum=d["mom"], second=d["sec"])])
    i32 = dict(dtype=torch.int32, device=DEV)
    fl = {k: torch.tensor([v], **i32) for k, v in dict(t=7, m=21, u=33, g=20).items()}
    status = torch.zeros(1, **i32)
    hyper = (33554, 9, 58982, 65470, 43980, 26)
    for kernel in ("momentum", "adam"):
        host = {k: [v[a:b].cpu().numpy().copy() for a, b in windows] for k, v in d.items()}
        if kernel == "momentum":
            lpk.lpk_momentum_sgd_step(tl, fl["t"], fl["t"], fl["m"], fl["m"], fl["g"], 6554, 58982, 0, None, None, status)
        else:
            lpk.lpk_adam_step(tl, fl["t"], fl["t"], fl["m"], fl["m"], fl["u"], fl["u"], fl["g"], hyper, None, None, None, status)
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        for w, (a, b) in enumerate(windows):
            th, co, mo, se, gr = (host[k][w] for k in ("theta", "comp", "mom", "sec", "grad"))
            if kernel == "momentum":
                ref.momentum_sgd_step(th, co, mo, gr, 7, 7, 7, 21, 21, 20, 6554, 58982, 0)
            else:
                ref.adam_step(th, co, mo, se, gr, 7, 7, 7, 21, 21, 33, 33, 20, *hyper)
            for k, want in (("theta", th), ("comp", co), ("mom", mo), ("sec", se)):
                assert np.array_equal(d[k][a:b].cpu().numpy(), want), (kernel, k, a, b)
        say("  %s: %d windows bit-exact" % (kernel, len(windows)))
    tl.destroy()

"""Momentum SGD with the lazy update inside: GPU library vs CPU oracle, bit for bit (needs an MI355X)."""
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

MU_Q16 = 58982        # RNE(0.9 * 2^16)
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


def compare(dev, host, what):
    th, co, fl_t, fl_g, vm, status = dev.download()
    assert status == int(host.status[0]), (what, "status")
    assert fl_t.tolist() == list(host.fl_theta) and fl_g.tolist() == list(host.fl_grad), (what, "fraclens")
    assert dev.fl_mom.cpu().tolist() == list(host.fl_mom), (what, "fl_mom", dev.fl_mom.cpu().tolist()[:8], host.fl_mom[:8])
    assert vm.tolist() == list(host.vmax), (what, "vmax")
    assert dev.mmax.cpu().numpy().view(np.uint64).tolist() == list(host.mmax), (what, "mmax")
    for t in range(host.cfg.n_tensors):
        assert np.array_equal(th[t], host.theta[t]), (what, "theta", t)
        assert np.array_equal(co[t], host.comp[t]), (what, "comp", t)
        assert np.array_equal(dev.mom[t].cpu().numpy(), host.mom[t]), (what, "mom", t)


def run_config(cfg, mom_bits, steps, fl_mom0=16, fused=False, comp_bits=None):
    from paper_1810_05486_amd.device_state import DeviceState
    dev = DeviceState(cfg, mom_bits=mom_bits, fl_mom0=fl_mom0, comp_bits=comp_bits)
    host = OracleState(cfg, mom_bits=mom_bits, fl_mom0=fl_mom0, comp_bits=comp_bits)
    views = dev.host_src_views()
    theta0 = [cfg.theta0(t, out=views[t]).copy() for t in range(cfg.n_tensors)]
    dev.upload_src()
    dev.init_theta()
    host.init_theta(theta0)
    for s in steps:
        grads = draw_grads(cfg, s, views)
        dev.upload_src()
        if fused:                                          # fp32 gradients straight into the update, no int16 round trip
            dev.select_grads()
            dev.update_momentum(cfg.lr_q16(s), MU_Q16, cfg.wd_q16, fused=True)
        else:
            dev.step(s, mu_q16=MU_Q16)
        host.step(s, grads, mu_q16=MU_Q16)
        compare(dev, host, "config %d step %d" % (cfg.id, s))
    dev.close()
    return host


def test_momentum_config1_int8_velocity():
    say("momentum: config 1, int8 velocity, 60 steps")
    host = run_config(workloads.config(1), [8], range(60))
    assert np.abs(host.mom[0].astype(int)).max() > 20          # the velocity grid settled and is being used


def test_momentum_lenet_int16_everything_reselect():
    say("momentum: LeNet shapes int16, int16 velocity, theta and velocity grids re-selected")
    cfg = workloads.config(2)
    run_config(cfg, [16] * cfg.n_tensors, range(40))


def test_momentum_resnet50_mixed_widths_decay():
    say("momentum: ResNet-50 shapes, int8 theta / int16 velocity (int16 classifier), weight decay")
    cfg = workloads.config(4)
    run_config(cfg, [16] * cfg.n_tensors, range(5))


def test_momentum_resnet18_int8_velocity():
    say("momentum: ResNet-18 shapes, all int8")
    cfg = workloads.config(3)
    run_config(cfg, [8] * cfg.n_tensors, [0, 1, 2, 3, 300, 600])


def test_momentum_config5_reduced():
    say("momentum: config 5 shape at reduced size")
    cfg = workloads.config(5, big_elems=(1 << 22) + 21, n_tiny=200)
    run_config(cfg, [8] * cfg.n_tensors, range(5))


@pytest.mark.parametrize("fused", [False, True])
def test_momentum_config5_full_size_in_bench_launch_configuration(fused):
    """The 1 Gi + 10000 x 256 workload at full size, the lists and launch shape `bench.py --momentum-bits 8` times
    (its int16-gradient step, then its fp32-gradient step), every output byte of two steps compared with the oracle
    (run on the host's threads)."""
    say("momentum: config 5 at FULL size, int8 velocity, 2 steps, fp32 gradients=%s" % fused)
    cfg = workloads.config(5)
    run_config(cfg, [8] * cfg.n_tensors, range(2), fused=fused)


@pytest.mark.parametrize("seed", fuzz_seeds(4))
def test_momentum_random_lists(seed):
    """Random widths, shifts, grid moves, alignments and sizes straight through the C ABI."""
    say("momentum: random lists, seed %d" % seed)
    rng = np.random.default_rng(500 + seed)
    pr = random.Random(600 + seed)
    sizes = [0, 1, 15, 16, 17, 255, 1024, 4095, 4096, 4097, 9001, 33000]
    for rep in range(8):
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
            delta_m = pr.choice([0, 0, 0, 0, 1, -1, pr.randint(-15, 15)])
            fl_m_out = fl_m_in + delta_m
            fl_g = fl_m_out + pr.choice([pr.randint(1, 14), pr.randint(1, 14), pr.randint(-20, 0), pr.randint(15, 50)])
            fls = [max(-64, min(64, f)) for f in (fl_in, fl_in + delta, fl_m_in, fl_m_out, fl_g)]
            n = pr.choice(sizes)
            mis = pr.choice([0, 0, 0, 1, 8, 16])
            c = dict(n=n, tb=tb, cb=cb, mb=mb, gb=gb, d=d, fls=fls)
            c["theta"] = rng.integers(-(2 ** (tb - 1)), 2 ** (tb - 1), size=n).astype(NP[tb])
            c["comp"] = rng.integers(-(2 ** (cb - 1)), 2 ** (cb - 1), size=n).astype(NP[cb]) if cb else None
            c["mom"] = rng.integers(-(2 ** (mb - 1)), 2 ** (mb - 1), size=n).astype(NP[mb])
            c["grad"] = rng.integers(-(2 ** (gb - 1)), 2 ** (gb - 1), size=n).astype(NP[gb])

            def dev(a, bits):
                buf = torch.zeros(n + 64, dtype=TT[bits], device=DEV)
                v = buf[mis:mis + n]
                v.copy_(torch.from_numpy(a))
                return buf, v
            c["bufs"] = []
            for key, bits in (("theta", tb), ("comp", cb), ("mom", mb), ("grad", gb)):
                if c[key] is None:
                    c["d_" + key] = None
                    continue
                b, v = dev(c[key], bits)
                c["bufs"].append(b); c["d_" + key] = v
            cases.append(c)
        lr_q, mu_q, wd_q = pr.choice([1, 655, 6554, 65535]), pr.choice([0, 58982, 65535, 32768]), pr.choice([0, 0, 7, 65535])
        tl = lpk.TensorList([lpk.make_desc(c["d_theta"], c["d_comp"], c["d_grad"], None,
                                           c["d"] if c["cb"] and c["d"] is not None else lpk.LPK_COMP_SHIFT_DEFAULT,
                                           momentum=c["d_mom"]) for c in cases])
        i32 = dict(dtype=torch.int32, device=DEV)
        arr = [torch.tensor([c["fls"][j] for c in cases], **i32) for j in range(5)]
        vmax = torch.full((len(cases),), 5, dtype=torch.int64, device=DEV)
        mmax = torch.full((len(cases),), 6, dtype=torch.int64, device=DEV)
        status = torch.zeros(1, dtype=torch.int32, device=DEV)
        lpk.lpk_momentum_sgd_step(tl, arr[0], arr[1], arr[2], arr[3], arr[4], lr_q, mu_q, wd_q, vmax, mmax, status)
        torch.cuda.synchronize()
        st = ref.new_status()
        for i, c in enumerate(cases):
            dd = c["d"] if c["d"] is not None else (c["cb"] - 1 if c["cb"] else 0)
            f = c["fls"]
            wv, wm = ref.momentum_sgd_step(c["theta"], c["comp"], c["mom"], c["grad"], dd, f[0], f[1], f[2], f[3], f[4],
                                           lr_q, mu_q, wd_q, st)
            ctx = {k: c[k] for k in ("n", "tb", "cb", "mb", "gb", "d", "fls")}
            ctx.update(lr=lr_q, mu=mu_q, wd=wd_q, i=i)
            assert np.array_equal(c["d_theta"].cpu().numpy(), c["theta"]), ("theta", ctx)
            if c["cb"]:
                assert np.array_equal(c["d_comp"].cpu().numpy(), c["comp"]), ("comp", ctx)
            assert np.array_equal(c["d_mom"].cpu().numpy(), c["mom"]), ("mom", ctx)
            assert int(vmax[i].item()) == wv and int(mmax[i].item()) == wm, ("max", ctx)
        assert int(status.cpu().numpy().view(np.uint32)[0]) == int(st[0])
        tl.destroy()


@pytest.mark.parametrize("store_all", [0, 1])
@pytest.mark.parametrize("tb,mb", [(8, 8), (8, 16), (16, 16)])
def test_momentum_runs_where_theta_moves_nowhere_somewhere_everywhere(tb, mb, store_all):
    """Gradients crafted so that, within one tensor, some wave-sized runs move no theta, some move one, some a dozen,
    some all of them; five steps with the velocity carrying over, every byte against the oracle, with and without
    LPK_OPT_STORE_ALL on the list (which must not change any result)."""
    say("momentum, theta moving in patches: theta int%d, velocity int%d, store_all=%d" % (tb, mb, store_all))
    rng = np.random.default_rng(500 + tb + mb + store_all)
    n = 40 * 4096 + 777
    theta = rng.integers(-100, 100, size=n).astype(NP[tb])
    comp = np.zeros(n, dtype=NP[tb]); mom = np.zeros(n, dtype=NP[mb])
    d = tb - 1
    fl_t, fl_g, fl_m = tb - 1, 15, (6 if mb == 8 else 14)
    d_theta, d_comp, d_mom = (torch.from_numpy(x).to(DEV) for x in (theta, comp, mom))
    d_grad = torch.zeros(n, dtype=torch.int16, device=DEV)
    tl = lpk.TensorList([lpk.make_desc(d_theta, d_comp, d_grad, None, momentum=d_mom)])
    lpk.lpk_tensor_list_set_option(tl, lpk.LPK_OPT_STORE_ALL, store_all)
    i32 = dict(dtype=torch.int32, device=DEV)
    a_t, a_g, a_m = torch.tensor([fl_t], **i32), torch.tensor([fl_g], **i32), torch.tensor([fl_m], **i32)
    vmax = torch.zeros(1, dtype=torch.int64, device=DEV); mmax = torch.zeros(1, dtype=torch.int64, device=DEV)
    status = torch.zeros(1, **i32)
    lr_q = 32768                                           # 1/2: a full-scale gradient moves theta by many LSBs
    moved = 0
    for step in range(5):
        g = np.zeros(n, dtype=np.int16)
        runs = n // 1024
        kind = rng.integers(0, 8, size=runs)              # most runs get no gradient (what moved before coasts on)
        for r in range(runs):
            lo = r * 1024
            if kind[r] == 5:   g[lo + int(rng.integers(0, 1024))] = 30000
            elif kind[r] == 6: g[lo + rng.choice(1024, size=12, replace=False)] = -30000
            elif kind[r] == 7: g[lo:lo + 1024] = rng.integers(-32768, 32767, size=1024)
        before = theta.copy()
        want_v, want_m = ref.momentum_sgd_step(theta, comp, mom, g, d, fl_t, fl_t, fl_m, fl_m, fl_g, lr_q, MU_Q16)
        moved += int((theta != before).sum())
        d_grad.copy_(torch.from_numpy(g))
        lpk.lpk_momentum_sgd_step(tl, a_t, a_t, a_m, a_m, a_g, lr_q, MU_Q16, 0, vmax, mmax, status)
        torch.cuda.synchronize()
        assert int(vmax.item()) == want_v and int(mmax.item()) == want_m and int(status.item()) == 0, step
        for name, dv, hv in (("theta", d_theta, theta), ("comp", d_comp, comp), ("mom", d_mom, mom)):
            bad = int((dv.cpu().numpy() != hv).sum())
            assert bad == 0, (step, name, bad)
    assert 0 < moved < 5 * n // 2                           # some theta moved, most did not
    tl.destroy()


def test_momentum_fused_fp32_gradient_step_equals_quantize_then_step():
    """lpk_momentum_sgd_step_f32grad against the oracle's quantize + momentum step, on every kind of workload."""
    say("fused momentum: config 1, int8 velocity")
    run_config(workloads.config(1), [8], range(40), fused=True)
    say("fused momentum: config 2 (int16 everything, grid moves)")
    cfg = workloads.config(2)
    run_config(cfg, [16] * cfg.n_tensors, range(40), fused=True)
    say("fused momentum: config 4 (mixed widths, decay, int16 velocity)")
    cfg = workloads.config(4)
    run_config(cfg, [16] * cfg.n_tensors, range(4), fused=True)
    say("fused momentum: config 5 reduced, ragged sizes, int8 then int16 velocity")
    cfg = workloads.config(5, big_elems=(1 << 22) + 37, n_tiny=300)
    run_config(cfg, [8] * cfg.n_tensors, range(4), fused=True)
    run_config(cfg, [16] * cfg.n_tensors, range(3), fused=True)


def test_momentum_fused_step_flags_non_finite_gradients():
    """NaN and +-Inf among the fp32 gradients: NaN quantizes to 0, Inf to the rails, the status word says so, and
    every other element goes on as usual -- as in the two-call sequence."""
    say("fused momentum: special gradient values")
    rng = np.random.default_rng(77)
    n = 3 * 4096 + 123
    theta = rng.integers(-100, 100, size=n).astype(np.int8); comp = rng.integers(-100, 100, size=n).astype(np.int8)
    mom = rng.integers(-3000, 3000, size=n).astype(np.int16)
    src = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    src[[5, 4096 + 17, n - 1]] = [np.nan, np.inf, -np.inf]
    fl_t, fl_m, fl_g = 7, 20, 18
    d_theta, d_comp, d_mom, d_src = (torch.from_numpy(x).to(DEV) for x in (theta, comp, mom, src))
    d_grad = torch.zeros(n, dtype=torch.int16, device=DEV)
    tl = lpk.TensorList([lpk.make_desc(d_theta, d_comp, d_grad, d_src, momentum=d_mom)])
    i32 = dict(dtype=torch.int32, device=DEV)
    a_t, a_m, a_g = torch.tensor([fl_t], **i32), torch.tensor([fl_m], **i32), torch.tensor([fl_g], **i32)
    vmax = torch.zeros(1, dtype=torch.int64, device=DEV); mmax = torch.zeros(1, dtype=torch.int64, device=DEV)
    status = torch.zeros(1, **i32)
    lpk.lpk_momentum_sgd_step_f32grad(tl, a_t, a_t, a_m, a_m, a_g, 6554, MU_Q16, 0, vmax, mmax, status)
    torch.cuda.synchronize()
    st = ref.new_status()
    g = ref.quantize(src, 16, fl_g, st)
    want_v, want_m = ref.momentum_sgd_step(theta, comp, mom, g, 7, fl_t, fl_t, fl_m, fl_m, fl_g, 6554, MU_Q16, 0, st)
    assert int(status.item()) == int(st[0]) and int(st[0]) & 1
    assert int(vmax.item()) == want_v and int(mmax.item()) == want_m
    assert np.array_equal(d_theta.cpu().numpy(), theta) and np.array_equal(d_comp.cpu().numpy(), comp)
    assert np.array_equal(d_mom.cpu().numpy(), mom)
    assert not d_grad.any().item()                          # the int16 gradient buffer was not touched
    tl.destroy()


@pytest.mark.parametrize("mb", [8, 16])
def test_momentum_all_int8_with_int8_gradients(mb):
    """The 8-bit training mode of Section 4 (int8 theta, accumulator and gradients, velocity int8 or int16) on the
    vector path: sparse and dense steps, weight decay, a velocity grid move, several tiles and a ragged tail, every byte
    against the oracle; then one step fed from fp32 gradients quantized to 8 bits in registers."""
    say("momentum: int8 theta, accumulator and gradients, int%d velocity" % mb)
    rng = np.random.default_rng(901)
    up = mb - 8                                            # a 16-bit velocity sits 8 bits finer
    n = 29 * 4096 + 4001
    theta = rng.integers(-100, 100, size=n).astype(np.int8); comp = rng.integers(-50, 50, size=n).astype(np.int8)
    mom = np.zeros(n, dtype=NP[mb])
    d_theta, d_comp, d_mom = (torch.from_numpy(x).to(DEV) for x in (theta, comp, mom))
    d_grad = torch.zeros(n, dtype=torch.int8, device=DEV); d_src = torch.zeros(n, dtype=torch.float32, device=DEV)
    tl = lpk.TensorList([lpk.make_desc(d_theta, d_comp, d_grad, d_src, momentum=d_mom)])
    i32 = dict(dtype=torch.int32, device=DEV)
    dev = lambda v: torch.tensor([v], **i32)
    vmax = torch.zeros(1, dtype=torch.int64, device=DEV); mmax = torch.zeros(1, dtype=torch.int64, device=DEV)
    status = torch.zeros(1, **i32)
    #        fl_m_in fl_m_out fl_g lr     wd  gradients
    plan = [(12,     12,      9,   655,   0,  "sparse"),
            (12,     12,      9,   6554,  0,  "dense"),
            (12,     11,      9,   6554,  7,  "dense"),
            (11,     11,      9,   655,   0,  "sparse")]
    for step, (fm_in, fm_out, fl_g, lr_q, wd_q, kind) in enumerate(plan):
        fm_in, fm_out = fm_in + up, fm_out + up
        g = rng.integers(-128, 128, size=n).astype(np.int8)
        if kind == "sparse":
            g[rng.random(n) > 0.002] = 0
        want_v, want_m = ref.momentum_sgd_step(theta, comp, mom, g, 7, 7, 7, fm_in, fm_out, fl_g, lr_q, MU_Q16, wd_q)
        d_grad.copy_(torch.from_numpy(g))
        lpk.lpk_momentum_sgd_step(tl, dev(7), dev(7), dev(fm_in), dev(fm_out), dev(fl_g), lr_q, MU_Q16, wd_q, vmax, mmax, status)
        torch.cuda.synchronize()
        assert int(vmax.item()) == want_v and int(mmax.item()) == want_m and int(status.item()) == 0, step
        for name, dv, hv in (("theta", d_theta, theta), ("comp", d_comp, comp), ("mom", d_mom, mom)):
            bad = int((dv.cpu().numpy() != hv).sum())
            assert bad == 0, (step, name, bad)
    assert int(np.abs(mom.astype(int)).max()) > 20 << up
    src = (rng.standard_normal(n) * 0.1).astype(np.float32)
    st = ref.new_status()
    g = ref.quantize(src, 8, 9, st)
    want_v, want_m = ref.momentum_sgd_step(theta, comp, mom, g, 7, 7, 7, 11 + up, 11 + up, 9, 6554, MU_Q16, 0, st)
    d_src.copy_(torch.from_numpy(src)); d_grad.zero_()
    lpk.lpk_momentum_sgd_step_f32grad(tl, dev(7), dev(7), dev(11 + up), dev(11 + up), dev(9), 6554, MU_Q16, 0, vmax, mmax, status)
    torch.cuda.synchronize()
    assert int(vmax.item()) == want_v and int(mmax.item()) == want_m and int(status.item()) == int(st[0]) == 0
    assert int(g.min()) == -128 and int(g.max()) == 127 and not d_grad.any().item()
    for dv, hv in ((d_theta, theta), (d_comp, comp), (d_mom, mom)):
        assert np.array_equal(dv.cpu().numpy(), hv)
    tl.destroy()


def test_momentum_int8_theta_with_int16_accumulator():
    """Section 2's 22-bit parameter (8-bit theta, 16-bit accumulator) under the momentum optimizer: ResNet-18 shapes
    and the reduced stress shape, int8 and int16 velocity, int16 and fp32 gradient sources."""
    cfg = workloads.config(3)
    say("momentum: int8 theta + int16 comp, config 3 shapes, int16 velocity")
    run_config(cfg, [16] * cfg.n_tensors, [0, 1, 2, 300, 600], comp_bits=[16] * cfg.n_tensors)
    cfg = workloads.config(5, big_elems=(1 << 22) + 9, n_tiny=100)
    say("momentum: int8 theta + int16 comp, config 5 reduced, int8 velocity, then fed from fp32 gradients")
    run_config(cfg, [8] * cfg.n_tensors, range(4), comp_bits=[16] * cfg.n_tensors)
    run_config(cfg, [16] * cfg.n_tensors, range(3), comp_bits=[16] * cfg.n_tensors, fused=True)


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
def test_momentum_random_workloads_follow_the_oracle_step_by_step(seed):
    """Random parameter sets through 30 consecutive momentum steps (velocity 8 or 16 bits wide per tensor, its grid
    re-selected every step with the one-step lag), plain or fed from the fp32 gradients; everything after every step."""
    pr = random.Random(4300 + seed)
    cfg = random_workload(pr, 200 + seed)
    mom_bits = [pr.choice([8, 16]) for _ in cfg.bits]
    fused = pr.random() < 0.4
    say("momentum: random workload %d: %d tensors, %d parameters, reselect=%s, fused=%s" % (seed, cfg.n_tensors, cfg.n_params,
                                                                                           cfg.reselect, fused))
    run_config(cfg, mom_bits, range(30), fl_mom0=pr.choice([16, 20, 24]), fused=fused)

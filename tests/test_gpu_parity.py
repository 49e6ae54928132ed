"""GPU library vs CPU oracle, bit for bit, through the C ABI (needs an MI355X)."""
import os
import sys

import random

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_1810_05486_amd import workloads
from oracle_state import OracleState, draw_grads


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def compare_scalars(dev, host, what):
    """fraclens, vmax and the status word only (cheap: checked after every step)."""
    torch.cuda.synchronize()
    assert dev.fl_theta.cpu().tolist() == list(host.fl_theta), (what, "fl_theta")
    assert dev.fl_grad.cpu().tolist() == list(host.fl_grad), (what, "fl_grad")
    assert dev.vmax.cpu().numpy().view(np.uint64).tolist() == list(host.vmax), (what, "vmax")
    assert int(dev.status.cpu().numpy().view(np.uint32)[0]) == int(host.status[0]), (what, "status")


def compare(dev, host, what, check_vmax=True):
    th, co, fl_t, fl_g, vm, status = dev.download()
    assert status == int(host.status[0]), (what, "status", status, int(host.status[0]))
    assert fl_t.tolist() == list(host.fl_theta), (what, "fl_theta")
    assert fl_g.tolist() == list(host.fl_grad), (what, "fl_grad")
    if check_vmax:
        assert vm.tolist() == list(host.vmax), (what, "vmax")
    for t in range(host.cfg.n_tensors):
        bad = int((th[t] != host.theta[t]).sum())
        assert bad == 0, (what, "theta", t, bad)
        if host.kahan:
            bad = int((co[t] != host.comp[t]).sum())
            assert bad == 0, (what, "comp", t, bad)


def run_config(cfg, step_ids, compare_every=1, kahan=True, always=(), comp_bits=None, fused=False, grad_bits=16, onepass=False):
    """A workload whose gradients cycle through a few draws (config 5) keeps every draw resident, in HBM and on the
    host, as bench.py does: from the second round of the cycle on a step costs no draw and no upload."""
    from paper_1810_05486_amd.device_state import DeviceState
    n_src = cfg.grad_cycle or 1
    dev = DeviceState(cfg, kahan=kahan, comp_bits=comp_bits, grad_bits=grad_bits, n_src=n_src)
    host = OracleState(cfg, kahan=kahan, comp_bits=comp_bits, grad_bits=grad_bits)
    views = dev.host_src_views()
    theta0 = [cfg.theta0(t, out=views[t]).copy() for t in range(cfg.n_tensors)]
    dev.upload_src()
    dev.init_theta()
    host.init_theta(theta0)
    del theta0
    compare(dev, host, "init", check_vmax=False)
    resident = {}
    for i, s in enumerate(step_ids):
        k = s % n_src
        if k in resident:
            grads = resident[k]
        else:
            grads = draw_grads(cfg, s, views)
            dev.upload_src(k)
            if cfg.grad_cycle:
                grads = resident[k] = [g.copy() for g in grads]
        if fused:
            dev.step_fused(s, k)
        else:
            dev.step(s, k, onepass=onepass(s) if callable(onepass) else onepass)
        host.step(s, grads)
        if (i + 1) % compare_every == 0 or i == len(step_ids) - 1 or i in always:
            compare(dev, host, "config %d step %d" % (cfg.id, s))
        else:
            compare_scalars(dev, host, "config %d step %d" % (cfg.id, s))
        if (i + 1) % 25 == 0:
            say("  config %d: %d/%d steps bit-exact so far" % (cfg.id, i + 1, len(step_ids)))
    if fused:                                   # the fused call never writes the int16 gradient arena
        assert int(dev.arena_grad.count_nonzero().item()) == 0
    dev.close()
    return host


def test_config1_single_tensor_100_steps():
    say("config 1: 65536 int8, 100 steps")
    host = run_config(workloads.config(1), range(100))
    assert host.fl_theta == [7]


def test_config1_without_accumulator():
    say("config 1 without the accumulator (plain SGD in int8)")
    run_config(workloads.config(1), range(20), kahan=False)


def test_config2_lenet_reselect():
    say("config 2: LeNet-5 shapes, int16, fraclen re-selected every step, all 1000 steps, every byte after each")
    run_config(workloads.config(2), range(1000))


def test_config3_resnet18_stepped_lr():
    """All 1000 steps, so the state follows the workload's own trajectory across both learning-rate drops: fraclens,
    vmax and status compared after every step, every byte every 50 steps and on the steps around the drops."""
    say("config 3: ResNet-18 shapes, int8, lr steps at 300 and 600, all 1000 steps")
    run_config(workloads.config(3), range(1000), compare_every=50, always=(0, 1, 299, 300, 301, 599, 600, 601))


def test_config4_resnet50_mixed_width_decay():
    say("config 4: ResNet-50 shapes, int8 + int16 classifier, weight decay, all 200 steps")
    run_config(workloads.config(4), range(200), compare_every=50, always=(0, 1, 2))


def test_config5_reduced():
    say("config 5 shape at reduced size: one 8 Mi + 37-element-ragged tensor and 300 tensors of 256")
    cfg = workloads.config(5, big_elems=(1 << 23) + 37, n_tiny=300)
    run_config(cfg, range(6))


def test_config5_full_size_in_bench_launch_configuration():
    """The headline workload at full size (1 Gi + 10000 x 256 elements), same lists and launch shape as bench.py.
    All 50 steps: every output byte compared with the oracle after steps 1, 2, 25 and 50, fraclens, vmax and status
    after every step; the first half through select + quantize, the second half (every other step of a shortened run)
    through lpk_select_quantize.  LPK_CONFIG5_STEPS=n shortens the run."""
    steps = int(os.environ.get("LPK_CONFIG5_STEPS", "50"))
    say("config 5 at FULL size: 1073741824 + 10000*256 elements, %d steps (oracle on host threads)" % steps)
    run_config(workloads.config(5), range(steps), compare_every=25, always=(0, 1),
               onepass=(lambda s: s >= 25) if steps >= 50 else (lambda s: s % 2 == 1))


def test_fused_fp32_gradient_step_equals_quantize_then_step():
    """lpk_kahan_sgd_step_f32grad against the oracle's quantize + update, on every kind of workload."""
    say("fused fp32-gradient update: config 1")
    run_config(workloads.config(1), range(40), fused=True)
    say("fused fp32-gradient update: config 2 (int16, grid moves)")
    run_config(workloads.config(2), range(60), fused=True)
    say("fused fp32-gradient update: config 4 (mixed widths, decay)")
    run_config(workloads.config(4), range(4), fused=True)
    say("fused fp32-gradient update: config 5 reduced")
    run_config(workloads.config(5, big_elems=(1 << 23) + 37, n_tiny=300), range(4), fused=True)
    say("fused fp32-gradient update: without the accumulator")
    run_config(workloads.config(1), range(10), fused=True, kahan=False)


def test_int8_theta_with_int16_accumulator():
    """The paper's 22-bit example (Section 2): 8-bit parameter, 16-bit accumulator, no overlapping bit (d = 15)."""
    say("int8 theta + int16 comp: config 3 shapes")
    cfg = workloads.config(3)
    run_config(cfg, [0, 1, 2, 300, 600], comp_bits=[16] * cfg.n_tensors)
    say("int8 theta + int16 comp: config 5 reduced, plain and fused")
    cfg = workloads.config(5, big_elems=(1 << 22) + 5, n_tiny=100)
    run_config(cfg, range(4), comp_bits=[16] * cfg.n_tensors)
    run_config(cfg, range(4), comp_bits=[16] * cfg.n_tensors, fused=True)


def test_all_8_bit_mode_whole_path():
    """Section 4's INT8 training with the lazy update: int8 parameters, accumulators and gradients.  The whole path
    (max-abs selection for an 8-bit grid, quantization to int8, update) on the single-tensor workload, the ResNet-18
    shapes and the reduced stress shape, plain and fed from the fp32 gradients."""
    say("all 8 bits: config 1, 60 steps")
    run_config(workloads.config(1), range(60), grad_bits=8)
    say("all 8 bits: config 3 (62 tensors, stepped learning rate)")
    run_config(workloads.config(3), [0, 1, 2, 300, 600], grad_bits=8)
    say("all 8 bits: config 5 reduced, plain and fused")
    cfg = workloads.config(5, big_elems=(1 << 22) + 77, n_tiny=100)
    run_config(cfg, range(4), grad_bits=8)
    run_config(cfg, range(4), grad_bits=8, fused=True)
    say("8-bit parameters and gradients with a 16-bit accumulator")
    run_config(cfg, range(3), grad_bits=8, comp_bits=[16] * cfg.n_tensors)


def test_selection_and_quantization_in_one_pass_on_every_workload():
    """lpk_select_quantize in place of select + quantize, with last step's fraclens as the guess: the first step's
    guess is the initial default (wrong for most tensors: quantized again), later ones mostly hold on the single-tensor
    and stress workloads and often fail on the small networks, whose maxima move from draw to draw; every byte, every
    fraclen and the status word after every step either way."""
    say("one-pass selection + quantization: config 1")
    run_config(workloads.config(1), range(30), onepass=True)
    say("one-pass selection + quantization: config 2 (int16, grid moves)")
    run_config(workloads.config(2), range(40), onepass=True)
    say("one-pass selection + quantization: config 3")
    run_config(workloads.config(3), range(12), onepass=True)
    say("one-pass selection + quantization: config 4 (mixed widths)")
    run_config(workloads.config(4), range(6), onepass=True)
    say("one-pass selection + quantization: config 5 reduced")
    run_config(workloads.config(5, big_elems=(1 << 23) + 37, n_tiny=300), range(7), onepass=True)
    say("one-pass selection + quantization: all 8 bits, config 5 reduced")
    run_config(workloads.config(5, big_elems=(1 << 22) + 77, n_tiny=100), range(4), onepass=True, grad_bits=8)


@pytest.mark.parametrize("fused", [False, True, "onepass"])
def test_whole_step_replayed_from_a_hip_graph(fused):
    """The hot calls only enqueue kernels, so a whole step (three calls, or two with the quantization fused into the
    update) can be recorded once and replayed: every replay (fresh gradients uploaded eagerly in between, a
    synchronization and a download after each) matches the oracle."""
    from paper_1810_05486_amd.device_state import DeviceState
    for cfg in (workloads.config(1), workloads.config(3), workloads.config(5, big_elems=(1 << 21) + 77, n_tiny=64)):
        say("hip graph replay: config %d, fused=%s" % (cfg.id, fused))
        dev, host = DeviceState(cfg), OracleState(cfg)
        views = dev.host_src_views()
        theta0 = [cfg.theta0(t, out=views[t]).copy() for t in range(cfg.n_tensors)]
        dev.upload_src()
        dev.init_theta()
        host.init_theta(theta0)
        grads = [cfg.grad(t, 0, out=views[t]) for t in range(cfg.n_tensors)]
        dev.upload_src()
        # runs step 0 eagerly once, then records it (recording executes nothing); "onepass": lpk_select_quantize + update
        graph = dev.capture_step(0, fused=fused is True, onepass=fused == "onepass")
        host.step(0, grads)
        compare(dev, host, "config %d eager step before the replays" % cfg.id)
        for s in range(1, 7):
            grads = draw_grads(cfg, s, views)
            dev.upload_src()
            graph.replay()
            host.step(s, grads)
            compare(dev, host, "config %d graph replay %d" % (cfg.id, s))
        del graph
        dev.close()


def fuzz_seeds(default_count):
    """Seeds of the random tests: 0..default_count-1, or LPK_FUZZ_SEEDS=lo:hi for a longer differential run."""
    spec = os.environ.get("LPK_FUZZ_SEEDS")
    if not spec:
        return range(default_count)
    lo, hi = (int(x) for x in spec.split(":"))
    return range(lo, hi)


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
def test_random_workloads_follow_the_oracle_step_by_step(seed):
    """Whole trajectories, not single calls: random parameter sets through 30 consecutive steps of select, quantize and
    update (or the fused update), with or without fraclen re-selection, weight decay, a 16-bit accumulator under
    8-bit parameters, or no accumulator at all; every byte and every scalar after every step."""
    pr = random.Random(4100 + seed)
    cfg = random_workload(pr, 100 + seed)
    kahan = pr.random() < 0.85
    comp_bits = [16 if b == 8 and pr.random() < 0.3 else b for b in cfg.bits] if kahan and pr.random() < 0.4 else None
    fused = pr.random() < 0.4
    onepass = not fused and pr.random() < 0.5          # lpk_select_quantize in place of select + quantize
    say("random workload %d: %d tensors, %d parameters, reselect=%s, kahan=%s, fused=%s, onepass=%s"
        % (seed, cfg.n_tensors, cfg.n_params, cfg.reselect, kahan, fused, onepass))
    run_config(cfg, range(30), kahan=kahan, comp_bits=comp_bits, fused=fused, onepass=onepass)

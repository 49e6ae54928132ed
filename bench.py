#!/usr/bin/env python3
"""Benchmark of the lazy-update hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 5]

A step is one pass of the whole path over one batch of synthetic fp32
gradients already resident in HBM: max-abs fraclen selection, quantization to
int16, the fused Kahan-SGD update with its vmax reduction (and the fraclen
re-selection where the workload has one).  Prints ONE JSON line.

  value         whole-path parameters per second (Gparam/s) over the K timed steps
  update_only   the same for lpk_kahan_sgd_step alone (the headline kernel)
  roofline      the update kernel against the 8 TB/s HBM peak.  `achieved` / `frac`: ALGORITHMIC bytes (6 B per
                int8 parameter, 10 B per int16 one) over the kernel's average duration, measured with HIP events
                around every call inside the timed region.  `traffic` / `frac_hbm`: the HBM bytes the kernel
                really moved per launch (it does not write back 16-byte groups a step leaves unchanged), from
                rocprofv3 FETCH_SIZE / WRITE_SIZE counters collected by this run in two child processes (scaled by
                the same counters on a plain copy of known size), over the same duration.
  regimes       the update kernel alone at learning rates where nothing changes, where few accumulators change
                (the workload's own), where most do, and with every store forced: time, frac and frac_hbm each
  ceilings      what the memory system gives plain reads, writes, a copy, and the update's own byte mix without
                arithmetic (libmembw, not part of the library's ABI)
  int16_update  the 16-bit parameter/accumulator path (10 B per parameter) on the same stress shape
  small_configs the launch-bound workloads 1-4: microseconds per step, eager and replayed from a HIP graph
  cpu_baseline  the CPU oracle on the host cores (and on one thread), on a bounded slice
"""
import argparse
import csv
import glob
import json
import os
import shutil
import signal
import statistics
import subprocess
import sys
import tempfile
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
REGIME_LRS = (("nothing_changes", 218), ("few_accumulators_change", 655), ("most_accumulators_change", 1310))
FLOOR_US = {1: 0.05, 2: 0.54, 3: 8.8, 4: 20.0}            # algorithmic bytes of one update at 8 TB/s


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def spread(ms):
    """mean / median / min of a list of per-launch times (ms)."""
    return {"mean": sum(ms) / len(ms), "median": statistics.median(ms), "min": min(ms)}


def timed(torch, fn, reps, warm=2):
    """Per-call times in ms: HIP events on the current stream (the one the library calls are launched on)."""
    for _ in range(warm):
        fn()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return [a.elapsed_time(b) for a, b in ev]


# ------------------------------------------------------------------------------------------ workload set-up

def make_config(args):
    from paper_1810_05486_amd import workloads
    cfg = workloads.config(args.config, big_elems=args.big_elems, n_tiny=args.n_tiny) if args.config == 5 else workloads.config(args.config)
    if args.lr_q16:
        cfg.lr_schedule = [(0, args.lr_q16)]
    if args.theta_bits:
        cfg.bits = [args.theta_bits] * cfg.n_tensors
    return cfg


def make_state(cfg, args, n_src):
    """Device arenas and lists for the workload, theta0 quantized in place, n_src gradient draws resident."""
    import torch
    from paper_1810_05486_amd.device_state import DeviceState
    mom_bits = [args.momentum_bits] * cfg.n_tensors if args.momentum_bits else None
    comp_bits = [args.comp_bits] * cfg.n_tensors if args.comp_bits else None
    if args.adam:
        mom_bits = [16] * cfg.n_tensors
    sec_bits = [16] * cfg.n_tensors if args.adam else None
    dev = DeviceState(cfg, n_src=n_src, mom_bits=mom_bits, comp_bits=comp_bits, sec_bits=sec_bits, fl_mom0=24, fl_sec0=38,
                      grad_bits=args.grad_bits)
    views = dev.host_src_views()
    t0 = time.perf_counter()
    for t in range(cfg.n_tensors):
        cfg.theta0(t, out=views[t])
    dev.upload_src(0)
    dev.init_theta(0)
    torch.cuda.synchronize()
    for k in range(n_src):
        for t in range(cfg.n_tensors):
            cfg.grad(t, k, out=views[t])
        dev.upload_src(k)
    torch.cuda.synchronize()
    log("workload %d: %d tensors, %d parameters; inputs drawn and uploaded in %.1f s (%d gradient draws resident)"
        % (cfg.id, cfg.n_tensors, cfg.n_params, time.perf_counter() - t0, n_src))
    return dev


def whole_step(dev, cfg, args, s, k, mu_q16):
    from paper_1810_05486_amd import workloads
    if args.adam:
        dev.quantize_grads(k)
        dev.update_adam(workloads.adam_hyper(s), k)
    else:
        dev.step(s, k=k, mu_q16=mu_q16)


def update_bytes(cfg, dev, args):
    b = sum(n * (2 * (tb // 8) + 2 * (cb // 8) + args.grad_bits // 8) for n, tb, cb in zip(cfg.sizes, cfg.bits, dev.comp_bits))
    b += 2 * (args.momentum_bits // 8) * cfg.n_params if args.momentum_bits else 0
    b += 8 * cfg.n_params if args.adam else 0
    return b


def kernel_names(args):
    """(update kernel, fused update kernel) as they appear in profiler output."""
    if args.adam:
        return "adam_step_kernel<0>", "adam_step_kernel<1>"
    if args.momentum_bits:
        return "momentum_step_kernel<0>", "momentum_step_kernel<1>"
    i8 = "true" if args.grad_bits == 8 else "false"
    return "kahan_step_kernel<0, false, %s>" % i8, "kahan_step_kernel<1, false, false>"


# ------------------------------------------------------------------------------------------ HBM traffic counters
#
# The parent (before it touches the GPU itself) runs this file twice under `rocprofv3 --pmc`, once per counter.
# The child sets the workload up exactly as the timed run does and launches a short, known sequence of kernels,
# writing that sequence ("plan") to a file; the parent matches the profiler's per-dispatch rows against the plan.

def traffic_child(args):
    import torch
    from paper_1810_05486_amd import binding as lpk
    from paper_1810_05486_amd import membw, workloads
    torch.cuda.set_device(0)
    cfg = make_config(args)
    plan = []                                                # (kernel-name substring, label) in launch order

    def note(kernel, label, n=1):
        plan.extend([(kernel, label)] * n)

    upd, fus = kernel_names(args)
    plain = not args.adam and not args.momentum_bits
    dev = make_state(cfg, args, 1)
    note("maxabs_f32_kernel", "init"); note("quantize_kernel", "init")
    mu_q16 = 58982 if args.momentum_bits else None
    for s in range(args.warmup):
        whole_step(dev, cfg, args, s, 0, mu_q16)
        note("maxabs_f32_kernel", "warmup"); note("quantize_kernel", "warmup"); note(upd, "warmup")
    copy = membw.Runner("copy", min(cfg.n_params, 1 << 30) // 16)
    for _ in range(3):
        copy.launch(4, 3)
    note("membw_kernel", "copy", 3)
    L = dev.lists[0]
    for _ in range(2):
        dev.quantize_grads(0)
        note("maxabs_f32_kernel", "maxabs"); note("quantize_kernel", "quantize")
    for _ in range(2):                                       # the fraclens just selected are the guess: it holds
        dev.quantize_grads_onepass(0)
        note("quantize_guess_kernel", "select_quantize")
    s0 = args.warmup
    if plain:
        for label, lr in REGIME_LRS:
            lr = cfg.lr_q16(s0) if label == "few_accumulators_change" else lr
            for _ in range(3):
                lpk.lpk_kahan_sgd_step(L, dev.fl_theta, dev.fl_next, dev.fl_grad, lr, cfg.wd_q16, dev.vmax, dev.status)
            note(upd, label, 3)
        lpk.lpk_tensor_list_set_option(L, lpk.LPK_OPT_STORE_ALL, 1)
        for _ in range(3):
            lpk.lpk_kahan_sgd_step(L, dev.fl_theta, dev.fl_next, dev.fl_grad, cfg.lr_q16(s0), cfg.wd_q16, dev.vmax, dev.status)
        note(upd.replace("<0, false", "<0, true"), "all_stores", 3)
        lpk.lpk_tensor_list_set_option(L, lpk.LPK_OPT_STORE_ALL, 0)
        for _ in range(2):
            lpk.lpk_kahan_sgd_step_f32grad(L, dev.fl_theta, dev.fl_next, dev.fl_grad, cfg.lr_q16(s0), cfg.wd_q16, dev.vmax, dev.status)
        note(fus, "fused", 2)
    else:
        for i in range(3):
            if args.adam:
                dev.update_adam(workloads.adam_hyper(s0 + i), 0)
            else:
                dev.update_momentum(cfg.lr_q16(s0), mu_q16, cfg.wd_q16, 0)
        note(upd, "update", 3)
        for i in range(2):
            if args.adam:
                dev.update_adam(workloads.adam_hyper(s0 + 3 + i), 0, fused=True)
            else:
                dev.update_momentum(cfg.lr_q16(s0), mu_q16, cfg.wd_q16, 0, fused=True)
        note(fus, "fused", 2)
    torch.cuda.synchronize()
    with open(args.traffic_child, "w") as f:
        json.dump({"plan": plan, "copy_bytes_each_way": copy.bytes_read}, f)
    dev.close()
    return 0


def _run_counter_pass(counter, args, workdir):
    """One `rocprofv3 --pmc <counter>` pass over the child; returns {label: mean counter value} and the copy size."""
    rocprof = shutil.which("rocprofv3") or "/opt/rocm/bin/rocprofv3"
    if not os.path.exists(rocprof):
        raise RuntimeError("rocprofv3 not found")
    out = os.path.join(workdir, counter.lower())
    plan_path = os.path.join(workdir, counter.lower() + "_plan.json")
    fwd = ["--config", str(args.config), "--big-elems", str(args.big_elems), "--n-tiny", str(args.n_tiny),
           "--warmup", str(args.warmup), "--grad-bits", str(args.grad_bits)]
    for flag, v in (("--lr-q16", args.lr_q16), ("--momentum-bits", args.momentum_bits), ("--comp-bits", args.comp_bits),
                    ("--theta-bits", args.theta_bits)):
        if v:
            fwd += [flag, str(v)]
    if args.adam:
        fwd.append("--adam")
    cmd = [rocprof, "--pmc", counter, "--output-format", "csv", "-d", out, "-o", "pmc", "--",
           sys.executable, os.path.join(ROOT, "bench.py"), "--traffic-child", plan_path] + fwd
    env = dict(os.environ, TMPDIR="/tmp")
    p = subprocess.Popen(cmd, cwd="/tmp", env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, start_new_session=True)
    try:
        text, _ = p.communicate(timeout=args.traffic_timeout)
    except subprocess.TimeoutExpired:
        os.killpg(p.pid, signal.SIGKILL)                    # the process group this call started, nothing else
        p.communicate()
        raise RuntimeError("rocprofv3 --pmc %s pass timed out after %d s" % (counter, args.traffic_timeout))
    if p.returncode != 0 or not os.path.exists(plan_path):
        raise RuntimeError("rocprofv3 --pmc %s pass failed (rc %s): %s" % (counter, p.returncode, text.decode(errors="replace")[-400:]))
    files = glob.glob(os.path.join(out, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise RuntimeError("rocprofv3 wrote no counter_collection.csv")
    meta = json.load(open(plan_path))
    rows = []
    for fn in files:
        for r in csv.DictReader(open(fn)):
            if r["Counter_Name"] == counter:
                rows.append((int(r["Dispatch_Id"]), r["Kernel_Name"], float(r["Counter_Value"])))
    rows.sort()
    per_kernel, cursor, values = {}, {}, {}
    for key in {k for k, _ in meta["plan"]}:
        per_kernel[key] = [v for _, name, v in rows if ("::" + key) in name]      # whole names: not requantize for quantize
        cursor[key] = 0
    for key, label in meta["plan"]:
        i = cursor[key]
        if i >= len(per_kernel[key]):
            raise RuntimeError("profiler saw %d dispatches of %s, the plan has more" % (len(per_kernel[key]), key))
        cursor[key] = i + 1
        values.setdefault(label if label in ("init", "warmup") else label + "|" + key, []).append(per_kernel[key][i])
    for key in per_kernel:
        if cursor[key] != len(per_kernel[key]):
            raise RuntimeError("profiler saw %d dispatches of %s, the plan has %d" % (len(per_kernel[key]), key, cursor[key]))
    return {k: sum(v) / len(v) for k, v in values.items() if "|" in k}, meta["copy_bytes_each_way"]


def measure_traffic(args):
    """HBM bytes per launch of the kernels of this mode: two profiler passes (FETCH_SIZE, then WRITE_SIZE), each
    scaled by what the same counter reads for the plain copy of known size.  None (with the reason logged) if the
    profiler is missing or a pass fails."""
    workdir = tempfile.mkdtemp(prefix="lpk_traffic_", dir="/tmp")
    try:
        t0 = time.perf_counter()
        fetch, nb = _run_counter_pass("FETCH_SIZE", args, workdir)
        write, _ = _run_counter_pass("WRITE_SIZE", args, workdir)
        fu = nb / fetch["copy|membw_kernel"]
        wu = nb / write["copy|membw_kernel"]
        out = {"fetch_unit_bytes": fu, "write_unit_bytes": wu, "kernels": {}}
        for key in fetch:
            label, kernel = key.split("|", 1)
            if label == "copy":
                continue
            rb, wb = fetch[key] * fu, write.get(key, 0.0) * wu
            out["kernels"][label] = {"kernel": kernel, "fetch_bytes": rb, "write_bytes": wb, "bytes": rb + wb}
        out["seconds"] = time.perf_counter() - t0
        log("HBM traffic counters collected in %.0f s (one FETCH_SIZE unit = %.0f B, one WRITE_SIZE unit = %.0f B)"
            % (out["seconds"], fu, wu))
        return out
    except Exception as e:                                  # the bench line then says where its traffic figure is from
        log("HBM traffic counters NOT collected: %s" % e)
        return None
    finally:
        shutil.rmtree(workdir, ignore_errors=True)


def stored_traffic(cfg_id):
    """The committed figures of an earlier profiler run (fallback when this run cannot collect counters)."""
    path = os.path.join(ROOT, "profiles", "traffic_config%d.json" % cfg_id)
    try:
        return json.load(open(path)), "stored: profiles/traffic_config%d.json" % cfg_id
    except Exception:
        return None, None


# ------------------------------------------------------------------------------------------ CPU oracle baseline

def cpu_baseline(cfg, sample_elems, threads, gbits=16):
    """Time the oracle (as it stands) on the first `sample_elems` elements of tensor 0: one whole-path step
    (max-abs fraclen selection, quantization, lazy update), with `threads` host threads over contiguous
    element ranges."""
    import numpy as np
    from oracle import ref
    n = cfg.sizes[0] if sample_elems >= cfg.sizes[0] else sample_elems
    bits = cfg.bits[0]
    dt = np.int8 if bits == 8 else np.int16
    theta0 = cfg.theta0(0, count=n)
    grad = cfg.grad(0, 0, count=n)
    fl_t = ref.select_fraclen_f32_mt(theta0, bits, bits - 1, threads=threads)
    theta = ref.quantize_mt(theta0, bits, fl_t, threads=threads)
    del theta0
    comp = np.zeros(n, dtype=dt)
    t0 = time.perf_counter()
    fl_g = ref.select_fraclen_f32_mt(grad, gbits, gbits - 1, threads=threads)
    g = ref.quantize_mt(grad, gbits, fl_g, threads=threads)
    ref.kahan_sgd_step_mt(theta, comp, g, bits - 1, fl_t, fl_t, fl_g, cfg.lr_q16(0), cfg.wd_q16, threads=threads)
    dt_s = time.perf_counter() - t0
    return {"value": n / dt_s / 1e9, "unit": "Gparam/s", "cores": threads,
            "cores_in_affinity_mask": len(os.sched_getaffinity(0)), "kind": "oracle",
            "sample": "one whole-path step (select + quantize + update) over the first %d elements of tensor 0, "
                      "%.1f s wall on %d thread%s" % (n, dt_s, threads, "" if threads == 1 else "s")}


# ------------------------------------------------------------------------------------------ secondary measurements

def measure_int16_update(args):
    """The 16-bit theta/comp path (10 algorithmic bytes per parameter) on the stress shape, update kernel alone."""
    import torch
    from paper_1810_05486_amd import binding as lpk
    a = argparse.Namespace(**vars(args))
    a.theta_bits, a.momentum_bits, a.adam, a.comp_bits, a.grad_bits, a.lr_q16 = 16, 0, False, 0, 16, 0
    cfg = make_config(a)
    dev = make_state(cfg, a, 1)
    for s in range(3):
        dev.step(s, k=0)
    L = dev.lists[0]
    nbytes = update_bytes(cfg, dev, a)

    def upd():
        lpk.lpk_kahan_sgd_step(L, dev.fl_theta, dev.fl_next, dev.fl_grad, cfg.lr_q16(3), cfg.wd_q16, dev.vmax, dev.status)

    out = {"workload": "config 5 shape with int16 theta and comp (fraclen 15 + 15)", "bytes_per_launch": nbytes}
    ms = timed(torch, upd, args.steps)
    out["lazy_stores"] = dict(spread(ms), frac=nbytes / (statistics.mean(ms) * 1e-3) / 1e9 / HBM_PEAK_GBS)
    lpk.lpk_tensor_list_set_option(L, lpk.LPK_OPT_STORE_ALL, 1)
    ms = timed(torch, upd, args.steps)
    out["all_stores"] = dict(spread(ms), frac=nbytes / (statistics.mean(ms) * 1e-3) / 1e9 / HBM_PEAK_GBS)
    out["unit"] = "ms"
    dev.close()
    del dev
    torch.cuda.empty_cache()
    return out


def measure_small_configs(args):
    """Workloads 1-4 (launch-bound: 0.05-20 us of HBM time per update): microseconds per whole step, eager and
    replayed from a HIP graph, three-call path and the fused two-call path."""
    import torch
    out = {}
    reps = max(args.steps, 50)
    for cid in (1, 2, 3, 4):
        a = argparse.Namespace(**vars(args))
        a.config, a.theta_bits, a.momentum_bits, a.adam, a.comp_bits, a.grad_bits, a.lr_q16 = cid, 0, 0, False, 0, 16, 0
        cfg = make_config(a)
        dev = make_state(cfg, a, 1)
        for s in range(5):
            dev.step(s)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(reps):
            dev.step(5 + s)
        torch.cuda.synchronize()
        eager = (time.perf_counter() - t0) / reps * 1e6
        t0 = time.perf_counter()
        for s in range(reps):
            dev.step_fused(5 + s)
        torch.cuda.synchronize()
        eager_fused = (time.perf_counter() - t0) / reps * 1e6
        t0 = time.perf_counter()
        for s in range(reps):
            dev.step(5 + s, onepass=True)
        torch.cuda.synchronize()
        eager_onepass = (time.perf_counter() - t0) / reps * 1e6
        r = {"params": cfg.n_params, "tensors": cfg.n_tensors, "eager_us": eager, "eager_fused_us": eager_fused,
             "eager_onepass_us": eager_onepass, "hbm_floor_us": FLOOR_US[cid]}
        if not cfg.reselect:                                 # re-selection rotates device arrays between steps
            for key, fused in (("graph_us", False), ("graph_fused_us", True)):
                g = dev.capture_step(5, fused=fused)
                g.replay()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(reps):
                    g.replay()
                torch.cuda.synchronize()
                r[key] = (time.perf_counter() - t0) / reps * 1e6
                del g
        out["config%d" % cid] = r
        dev.close()
        del dev
    torch.cuda.empty_cache()
    return out


def measure_ceilings(args, n_params, mode_mix):
    """libmembw yardsticks at the headline size: best launch shape of 1, 2, 4 workgroups per CU x 1-8 groups."""
    import torch
    from paper_1810_05486_amd import membw
    units = min(n_params, 1 << 30) // 16
    out = {"unit": "GB/s", "note": "median of %d launches, best of 1/2/4 workgroups per CU and 1/2/4/8 groups in flight; "
                                   "no arithmetic, same accesses as the kernels (libmembw, outside the library's ABI)" % 10}
    for name in ("read", "write", "copy", "quantize", mode_mix):
        r = membw.Runner(name, units)
        best = max((r.best(b) + (b,)) for b in (1, 2, 4))
        out[r.name] = {"GB/s": best[0], "groups": best[1], "workgroups_per_cu": best[2], "frac_of_peak": best[0] / HBM_PEAK_GBS,
                       "bytes_read": r.bytes_read, "bytes_written": r.bytes_written}
        del r
        torch.cuda.empty_cache()
    return out


# ------------------------------------------------------------------------------------------ main

def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, help="workload 1..5 (5 = the 1 Gi-parameter headline)")
    ap.add_argument("--big-elems", type=int, default=1 << 30, help="size of config 5's large tensor")
    ap.add_argument("--n-tiny", type=int, default=10000, help="number of 256-element tensors in config 5")
    ap.add_argument("--lr-q16", type=int, default=0,
                    help="override the workload's Q0.16 learning rate (a larger step makes more parameters change per update)")
    ap.add_argument("--momentum-bits", type=int, default=0, choices=[0, 8, 16],
                    help="time the momentum variant of the update (velocity of this width, mu = 0.9) instead of plain SGD")
    ap.add_argument("--adam", action="store_true",
                    help="time the ADAM variant of the update (int16 first and second moments) instead of plain SGD")
    ap.add_argument("--grad-bits", type=int, default=16, choices=[8, 16],
                    help="width of the quantized gradients (8: the all-8-bit mode; not with --adam)")
    ap.add_argument("--comp-bits", type=int, default=0, choices=[0, 8, 16],
                    help="width of the accumulator when it differs from theta's (16 = the paper's 8+16 -> 22-bit example)")
    ap.add_argument("--theta-bits", type=int, default=0, choices=[0, 8, 16],
                    help="override the width of every parameter tensor (16: the int16 path on the chosen shape)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-traffic", action="store_true", help="do not run the two rocprofv3 counter passes")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the secondary measurements (regimes, ceilings, int16 path, small configs, graph replay)")
    ap.add_argument("--traffic-timeout", type=int, default=150, help="seconds allowed per rocprofv3 counter pass")
    ap.add_argument("--traffic-child", default="", help=argparse.SUPPRESS)
    ap.add_argument("--write-traffic", default="", help="also write the measured traffic figures to this JSON file")
    ap.add_argument("--cpu-sample", type=int, default=1 << 30,
                    help="elements of the oracle's all-threads sample (the one-thread sample is a quarter of it)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the update is elementwise and shards without "
                 "communication); --gpus %d is not supported." % args.gpus)
    if args.traffic_child:
        return traffic_child(args)

    # Counter passes first: the child processes are started before this process initialises the GPU.  Importing torch
    # (no GPU call yet) pages the libraries in, so that on a fresh machine the children do not spend their time limit
    # on that.
    import torch
    traffic = None if args.no_traffic else measure_traffic(args)

    from paper_1810_05486_amd import workloads
    from paper_1810_05486_amd import binding as lpk

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the hot path has no CPU fallback.")
    torch.cuda.set_device(0)

    cfg = make_config(args)
    n_src = cfg.grad_cycle or 3                     # timing only: cycle three resident gradient draws
    mu_q16 = 58982 if args.momentum_bits else None
    plain = mu_q16 is None and not args.adam
    dev = make_state(cfg, args, n_src)

    for s in range(args.warmup):
        whole_step(dev, cfg, args, s, s % n_src, mu_q16)
    torch.cuda.synchronize()

    # ---- the timed region: K whole steps, HIP events around each stage
    K = args.steps
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(K)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        s = args.warmup + i
        k = s % n_src
        ev[i][0].record()
        L = dev.lists[k]
        lpk.lpk_select_fraclen(L, lpk.LPK_F32, lpk.LPK_SEL_GRAD, None, None, dev.fl_grad, dev.fl_grad, dev.status)
        ev[i][1].record()
        lpk.lpk_quantize_tensor(L, lpk.LPK_SEL_GRAD, dev.fl_grad, dev.status)
        ev[i][2].record()
        if args.adam:
            dev.update_adam(workloads.adam_hyper(s), k)
        elif mu_q16 is None:
            dev.update(cfg.lr_q16(s), cfg.wd_q16, k)
        else:
            dev.update_momentum(cfg.lr_q16(s), mu_q16, cfg.wd_q16, k)
        ev[i][3].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    sel = [e[0].elapsed_time(e[1]) for e in ev]
    qnt = [e[1].elapsed_time(e[2]) for e in ev]
    upd = [e[2].elapsed_time(e[3]) for e in ev]
    sel_ms, qnt_ms, upd_ms = (sum(x) / K for x in (sel, qnt, upd))
    ms_per_step = wall * 1e3 / K

    # ---- the same whole path with quantization fused into the update (select + the optimizer's *_f32grad call)
    def fused_update(s, k):
        if args.adam:
            dev.update_adam(workloads.adam_hyper(s), k, fused=True)
        elif mu_q16 is not None:
            dev.update_momentum(cfg.lr_q16(s), mu_q16, cfg.wd_q16, k, fused=True)
        else:
            lpk.lpk_kahan_sgd_step_f32grad(dev.lists[k], dev.fl_theta, dev.fl_next, dev.fl_grad, cfg.lr_q16(s), cfg.wd_q16,
                                           dev.vmax, dev.status)
    fev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(K)]
    for s in range(2):
        dev.select_grads(s % n_src)
        fused_update(s, s % n_src)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(K):
        s = args.warmup + K + i
        k = s % n_src
        fev[i][0].record()
        dev.select_grads(k)
        fev[i][1].record()
        fused_update(s, k)
        fev[i][2].record()
    torch.cuda.synchronize()
    fwall = time.perf_counter() - t1
    f_upd = [e[1].elapsed_time(e[2]) for e in fev]

    # ---- the whole path with selection and quantization in one pass (lpk_select_quantize: last step's fraclens are the
    #      guess; the int16 gradients are written as in the three-call path), then the same update
    def plain_update(s, k):
        if args.adam:
            dev.update_adam(workloads.adam_hyper(s), k)
        elif mu_q16 is None:
            dev.update(cfg.lr_q16(s), cfg.wd_q16, k)
        else:
            dev.update_momentum(cfg.lr_q16(s), mu_q16, cfg.wd_q16, k)
    oev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(K)]
    for s in range(2):
        dev.quantize_grads_onepass(s % n_src)
        plain_update(s, s % n_src)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(K):
        s = args.warmup + 2 * K + i
        k = s % n_src
        oev[i][0].record()
        dev.quantize_grads_onepass(k)
        oev[i][1].record()
        plain_update(s, k)
        oev[i][2].record()
    torch.cuda.synchronize()
    owall = time.perf_counter() - t1
    o_sq = [e[0].elapsed_time(e[1]) for e in oev]
    sq_bytes = (4 + args.grad_bits // 8) * cfg.n_params
    onepass = {"value": cfg.n_params / (owall / K) / 1e9, "unit": "Gparam/s", "ms_per_step": owall * 1e3 / K,
               "stage_ms": {"select_quantize": statistics.mean(o_sq), "update": sum(e[1].elapsed_time(e[2]) for e in oev) / K},
               "select_quantize_ms": dict(spread(o_sq), max=max(o_sq)),
               "roofline": {"bound": "hbm", "kernel": "quantize_guess_kernel", "bytes_per_launch": sq_bytes, "peak": HBM_PEAK_GBS,
                            "unit": "GB/s", "achieved": sq_bytes / (statistics.mean(o_sq) * 1e-3) / 1e9,
                            "frac": sq_bytes / (statistics.mean(o_sq) * 1e-3) / 1e9 / HBM_PEAK_GBS,
                            "traffic": (traffic or {}).get("kernels", {}).get("select_quantize", {}).get("bytes")},
               "note": "same outputs as the three-call path (fraclens, int gradients, update); every guess held in these steps "
                       "unless select_quantize_ms.max stands out: a wrong guess costs that tensor one more quantization pass"}
    f_upd_ms = sum(f_upd) / K
    upd_kernel, fus_kernel = kernel_names(args)
    nbytes = update_bytes(cfg, dev, args)
    fbytes = nbytes + (4 - args.grad_bits // 8) * cfg.n_params
    tk = traffic["kernels"] if traffic else {}

    def frac_hbm(label, ms):
        return tk[label]["bytes"] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS if label in tk else None

    fused = {"value": cfg.n_params / (fwall / K) / 1e9, "unit": "Gparam/s", "ms_per_step": fwall * 1e3 / K,
             "stage_ms": {"select_fraclen": sum(e[0].elapsed_time(e[1]) for e in fev) / K, "kahan_sgd_step_f32grad": f_upd_ms},
             "roofline": {"bound": "hbm", "kernel": fus_kernel, "achieved": fbytes / (f_upd_ms * 1e-3) / 1e9,
                          "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": fbytes / (f_upd_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                          "traffic": tk.get("fused", {}).get("bytes"), "frac_hbm": frac_hbm("fused", f_upd_ms),
                          "bytes_per_launch": fbytes, "duration_ms": spread(f_upd)}}

    # ---- the update alone in four regimes of the lazy stores (the int16 gradients of the last step stay in place)
    regimes = all_stores = None
    if plain and not args.no_extras:
        regimes = {}
        L = dev.lists[(args.warmup + K - 1) % n_src]
        for label, lr in REGIME_LRS:
            lr = cfg.lr_q16(args.warmup) if label == "few_accumulators_change" else lr
            ms = timed(torch, lambda: lpk.lpk_kahan_sgd_step(L, dev.fl_theta, dev.fl_next, dev.fl_grad, lr, cfg.wd_q16,
                                                             dev.vmax, dev.status), K)
            m = statistics.mean(ms)
            regimes[label] = dict(spread(ms), lr_q16=lr, frac=nbytes / (m * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                  traffic=tk.get(label, {}).get("bytes"), frac_hbm=frac_hbm(label, m))
        lpk.lpk_tensor_list_set_option(L, lpk.LPK_OPT_STORE_ALL, 1)
        ms = timed(torch, lambda: lpk.lpk_kahan_sgd_step(L, dev.fl_theta, dev.fl_next, dev.fl_grad, cfg.lr_q16(args.warmup),
                                                         cfg.wd_q16, dev.vmax, dev.status), K)
        lpk.lpk_tensor_list_set_option(L, lpk.LPK_OPT_STORE_ALL, 0)
        m = statistics.mean(ms)
        regimes["all_stores"] = dict(spread(ms), lr_q16=cfg.lr_q16(args.warmup), frac=nbytes / (m * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                     traffic=tk.get("all_stores", {}).get("bytes"), frac_hbm=frac_hbm("all_stores", m))
        regimes["unit"] = "ms"
        a_gbs = nbytes / (m * 1e-3) / 1e9
        all_stores = {"bound": "hbm", "kernel": upd_kernel.replace("<0, false", "<0, true") + " (LPK_OPT_STORE_ALL)", "achieved": a_gbs,
                      "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": a_gbs / HBM_PEAK_GBS, "traffic": tk.get("all_stores", {}).get("bytes"),
                      "frac_hbm": frac_hbm("all_stores", m), "bytes_per_launch": nbytes, "ms": m}

    # ---- the same whole step replayed from HIP graphs (one recording per resident gradient draw)
    graph = None
    if plain and not cfg.reselect and not args.no_extras:
        graph = {}
        for key, fused_flag in (("ms_per_step", False), ("fused_ms_per_step", True)):
            graphs = [dev.capture_step(args.warmup, k, fused=fused_flag) for k in range(n_src)]
            for g in graphs:
                g.replay()
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            for i in range(K):
                graphs[i % n_src].replay()
            torch.cuda.synchronize()
            graph[key] = (time.perf_counter() - t2) * 1e3 / K
            del graphs
        graph["value"] = cfg.n_params / (graph["ms_per_step"] * 1e-3) / 1e9
        graph["fused_value"] = cfg.n_params / (graph["fused_ms_per_step"] * 1e-3) / 1e9
        graph["unit"] = "Gparam/s"

    status = int(dev.status.cpu().numpy().view("uint32")[0])
    dev.close()
    del dev
    torch.cuda.empty_cache()

    # ---- headline roofline object
    achieved = nbytes / (upd_ms * 1e-3) / 1e9
    label = "few_accumulators_change" if plain else "update"
    traffic_bytes = tk.get(label, {}).get("bytes")
    traffic_source = "measured in this run: rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE passes over the same workload, scaled by a plain copy of known size" if traffic_bytes else None
    if traffic_bytes is None and not args.lr_q16 and args.grad_bits == 16 and not args.comp_bits and not args.theta_bits:
        tj, src = stored_traffic(cfg.id)
        if tj:
            traffic_bytes = tj.get(upd_kernel.split("<")[0] + "_bytes_per_launch")
            traffic_source = "%s (%s)" % (src, tj.get("measured_at", "earlier run")) if traffic_bytes else None
    roofline = {"bound": "hbm", "kernel": upd_kernel, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": traffic_bytes,
                "frac_hbm": (traffic_bytes / (upd_ms * 1e-3) / 1e9 / HBM_PEAK_GBS) if traffic_bytes else None,
                "traffic_GB/s": (traffic_bytes / (upd_ms * 1e-3) / 1e9) if traffic_bytes else None,
                "traffic_fetch": tk.get(label, {}).get("fetch_bytes"), "traffic_write": tk.get(label, {}).get("write_bytes"),
                "traffic_source": traffic_source, "bytes_per_launch": nbytes, "duration_ms": spread(upd),
                "reading": ("`frac` is algorithmic bytes over time, as the benchmark contract defines it; the kernel does not "
                            "write back 16-byte groups of theta / comp that a step leaves unchanged (the lazy update's usual "
                            "case), so it moves fewer bytes than that: `frac_hbm` = measured HBM traffic over the same time is "
                            "the utilisation of the memory system, and `regimes.all_stores` is the same kernel writing every byte")
                           if plain else
                           ("the ADAM kernel sits where two bounds meet: its exact arithmetic and its in-place byte mix "
                            "(8 read : 6 written per parameter)" if args.adam else None)}

    out = {
        "metric": "Kahan-SGD update Gparams/s + achieved HBM GB/s (% of peak), 1 MI355X",
        "metric_note": "value = parameters per second over whole steps (max-abs fraclen selection + quantization to int16 + "
                       "fused Kahan update with vmax), fp32 gradients resident in HBM; update_only and roofline = the update kernel alone",
        "value": cfg.n_params / (ms_per_step * 1e-3) / 1e9,
        "unit": "Gparam/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "storage": "int8/int16 dynamic fixed point (32-bit integer + FMA-rounded arithmetic on the fast path, exact fp64 arithmetic elsewhere)",
        "config": {"workload": "config %d: %s%s" % (cfg.id, cfg.name, ", momentum 0.9 with int%d velocity" % args.momentum_bits
                                                    if args.momentum_bits else "") + (", ADAM with int16 moments" if args.adam else "")
                               + (", int%d accumulator" % args.comp_bits if args.comp_bits else "")
                               + (", int8 gradients" if args.grad_bits == 8 else "")
                               + (", every tensor int%d" % args.theta_bits if args.theta_bits else ""),
                   "n_tensors": cfg.n_tensors, "n_params": cfg.n_params, "lr_q16": cfg.lr_q16(0), "wd_q16": cfg.wd_q16,
                   "grad_draws_cycled": n_src},
        "update_only": {"value": cfg.n_params / (upd_ms * 1e-3) / 1e9, "unit": "Gparam/s", "ms": upd_ms},
        "stage_ms": {"select_fraclen": sel_ms, "quantize": qnt_ms, "kahan_sgd_step": upd_ms},
        "stage_ms_spread": {"select_fraclen": spread(sel), "quantize": spread(qnt), "kahan_sgd_step": spread(upd)},
        "roofline": roofline,
        "roofline_all_stores": all_stores,
        "regimes": regimes,
        "other_kernels": {
            "maxabs_f32_kernel": {"GB/s": 4 * cfg.n_params / (sel_ms * 1e-3) / 1e9, "bytes_per_launch": 4 * cfg.n_params,
                                  "frac": 4 * cfg.n_params / (sel_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                  "traffic": tk.get("maxabs", {}).get("bytes")},
            "quantize_kernel": {"GB/s": (4 + args.grad_bits // 8) * cfg.n_params / (qnt_ms * 1e-3) / 1e9,
                                "bytes_per_launch": (4 + args.grad_bits // 8) * cfg.n_params,
                                "frac": (4 + args.grad_bits // 8) * cfg.n_params / (qnt_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                "traffic": tk.get("quantize", {}).get("bytes")}},
        "fused_path": fused,
        "onepass_path": onepass,
        "graph_replay": graph,
        "device_status_word": status,
    }
    if traffic:
        out["traffic_counters"] = {"fetch_unit_bytes": traffic["fetch_unit_bytes"], "write_unit_bytes": traffic["write_unit_bytes"],
                                   "seconds": traffic["seconds"], "kernels": tk}
    if args.write_traffic and traffic:
        head = subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], capture_output=True, text=True).stdout.strip()
        base = upd_kernel.split("<")[0]
        rec = {"measured_at": "commit %s, %s" % (head or "unknown", time.strftime("%Y-%m-%d")),
               "command": "python bench.py " + " ".join(a for a in sys.argv[1:]),
               "workload": out["config"]["workload"], "lr_q16": cfg.lr_q16(0),
               "fetch_unit_bytes": traffic["fetch_unit_bytes"], "write_unit_bytes": traffic["write_unit_bytes"],
               base + "_bytes_per_launch": traffic_bytes, "kernels": tk}
        with open(args.write_traffic, "w") as f:
            json.dump(rec, f, indent=1)

    if not args.no_extras:
        mode_mix = "adam_i16" if args.adam else ({8: "momentum_i8v", 16: "momentum_i16v"}[args.momentum_bits] if args.momentum_bits
                                                else ("update_i16" if args.theta_bits == 16 else
                                                      ("update_i8_c16" if args.comp_bits == 16 else "update_i8")))
        out["ceilings"] = measure_ceilings(args, cfg.n_params, mode_mix)
        mix_gbs = [v["GB/s"] for k, v in out["ceilings"].items() if isinstance(v, dict) and k.startswith(mode_mix)]
        if mix_gbs and plain and regimes:
            out["ceilings"]["all_stores_kernel_over_its_mix"] = (nbytes / (regimes["all_stores"]["mean"] * 1e-3) / 1e9) / mix_gbs[0]
        elif mix_gbs:
            out["ceilings"]["update_kernel_over_its_mix"] = achieved / mix_gbs[0]
        c = out["ceilings"]
        qmix = [v["GB/s"] for k, v in c.items() if isinstance(v, dict) and k.startswith("quantize")]
        if qmix and args.grad_bits == 16:
            c["quantize_kernel_over_its_mix"] = out["other_kernels"]["quantize_kernel"]["GB/s"] / qmix[0]
        c["maxabs_kernel_over_read"] = out["other_kernels"]["maxabs_f32_kernel"]["GB/s"] / c["read"]["GB/s"]
        if plain and args.config == 5 and not args.theta_bits and not args.comp_bits and args.grad_bits == 16:
            out["int16_update"] = measure_int16_update(args)
            out["small_configs"] = measure_small_configs(args)
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a bounded sample ...")
        # host threads: this process's CPU share -- the GPU machine gives a one-GPU job 16 CPUs, whatever the affinity mask says
        cores = max(1, min(16, len(os.sched_getaffinity(0))))
        out["cpu_baseline"] = cpu_baseline(cfg, args.cpu_sample, cores, args.grad_bits)
        out["cpu_baseline_one_thread"] = cpu_baseline(cfg, args.cpu_sample // 4, 1, args.grad_bits)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())

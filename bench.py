#!/usr/bin/env python3
"""Benchmark of the lazy-update hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 5]

A step is one pass of the whole path over one batch of synthetic fp32
gradients already resident in HBM: max-abs fraclen selection, quantization to
int16, the fused Kahan-SGD update with its vmax reduction (and the fraclen
re-selection where the workload has one).  Prints ONE JSON line.

  value      whole-path parameters per second (Gparam/s) over the K timed steps
  update_only   the same for lpk_kahan_sgd_step alone (the headline kernel)
  roofline   the update kernel against the 8 TB/s HBM peak: algorithmic bytes
             (6 B per int8 parameter, 10 B per int16 one) over its average
             duration, measured with HIP events around every call inside the
             timed region
  cpu_baseline   the CPU oracle on the host cores (and on one thread), on a bounded slice
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def cpu_baseline(cfg, sample_elems, threads, gbits=16):
    """Time the oracle (as it stands) on the first `sample_elems` elements of tensor 0: one whole-path step
    (max-abs fraclen selection, quantization, lazy update), with `threads` host threads over contiguous
    element ranges (the selection scan stays on one thread, as the oracle has it)."""
    import numpy as np
    from oracle import ref
    n = cfg.sizes[0] if sample_elems >= cfg.sizes[0] else sample_elems
    bits = cfg.bits[0]
    dt = np.int8 if bits == 8 else np.int16
    theta0 = cfg.theta0(0, count=n)
    grad = cfg.grad(0, 0, count=n)
    fl_t = ref.select_fraclen_f32(theta0, bits, bits - 1)
    theta = ref.quantize(theta0, bits, fl_t)
    comp = np.zeros(n, dtype=dt)
    t0 = time.perf_counter()
    fl_g = ref.select_fraclen_f32(grad, gbits, gbits - 1)
    g = ref.quantize_mt(grad, gbits, fl_g, threads=threads)
    ref.kahan_sgd_step_mt(theta, comp, g, bits - 1, fl_t, fl_t, fl_g, cfg.lr_q16(0), cfg.wd_q16, threads=threads)
    dt_s = time.perf_counter() - t0
    return {"value": n / dt_s / 1e9, "unit": "Gparam/s", "cores": threads, "kind": "oracle",
            "sample": "one whole-path step (select + quantize + update) over the first %d elements of tensor 0, "
                      "%.1f s" % (n, dt_s)}


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
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-gib", type=float, default=2.0,
                    help="size of the plain-copy yardstick (lpk_stream_copy), 0 = skip")
    ap.add_argument("--cpu-sample", type=int, default=1 << 29,
                    help="elements of the oracle's all-threads sample (the one-thread sample is a quarter of it)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the update is elementwise and shards without "
                 "communication); --gpus %d is not supported." % args.gpus)

    import torch
    from paper_1810_05486_amd import workloads
    from paper_1810_05486_amd.device_state import DeviceState
    from paper_1810_05486_amd import binding as lpk

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the hot path has no CPU fallback.")
    torch.cuda.set_device(0)

    cfg = workloads.config(args.config, big_elems=args.big_elems, n_tiny=args.n_tiny) if args.config == 5 else workloads.config(args.config)
    if args.lr_q16:
        cfg.lr_schedule = [(0, args.lr_q16)]
    n_src = cfg.grad_cycle or 1
    if not cfg.grad_cycle:
        n_src = 3                                   # timing only: cycle three resident gradient draws
    log("workload %d: %s; %d tensors, %d parameters" % (cfg.id, cfg.name, cfg.n_tensors, cfg.n_params))
    mom_bits = [args.momentum_bits] * cfg.n_tensors if args.momentum_bits else None
    mu_q16 = 58982 if args.momentum_bits else None
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
        log("gradient draw %d/%d resident" % (k + 1, n_src))
    torch.cuda.synchronize()
    log("inputs drawn and uploaded in %.1f s" % (time.perf_counter() - t0))

    for s in range(args.warmup):
        if args.adam:
            dev.quantize_grads(s % n_src)
            dev.update_adam(workloads.adam_hyper(s), s % n_src)
        else:
            dev.step(s, k=s % n_src, mu_q16=mu_q16)
    torch.cuda.synchronize()

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

    # the same whole path with quantization fused into the update (select + the optimizer's *_f32grad call)
    fused = None
    if True:
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
        f_upd_ms = sum(e[1].elapsed_time(e[2]) for e in fev) / K
        fbytes = sum(n * (4 * (b // 8 + (cb // 8)) // 2 + 4) for n, b, cb in zip(cfg.sizes, cfg.bits, dev.comp_bits))
        fbytes += 2 * (args.momentum_bits // 8) * cfg.n_params if args.momentum_bits else 0
        fbytes += 8 * cfg.n_params if args.adam else 0
        fname = "adam_step_kernel<fp32 grad>" if args.adam else ("momentum_step_kernel<fp32 grad>" if args.momentum_bits else "kahan_step_kernel<fp32 grad>")
        fused = {"value": cfg.n_params / (fwall / K) / 1e9, "unit": "Gparam/s", "ms_per_step": fwall * 1e3 / K,
                 "stage_ms": {"select_fraclen": sum(e[0].elapsed_time(e[1]) for e in fev) / K, "kahan_sgd_step_f32grad": f_upd_ms},
                 "roofline": {"bound": "hbm", "kernel": fname, "achieved": fbytes / (f_upd_ms * 1e-3) / 1e9,
                              "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": fbytes / (f_upd_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                              "bytes_per_launch": fbytes}}

    # the update alone with LPK_OPT_STORE_ALL: every result written, changed or not (the int16 gradients of the last
    # step are still in place) -- the figure to read against the HBM roofline as a dense read-modify-write stream
    all_stores = None
    if mu_q16 is None and not args.adam:
        for L in dev.lists:
            lpk.lpk_tensor_list_set_option(L, lpk.LPK_OPT_STORE_ALL, 1)
        aev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(K)]
        for i in range(K + 2):
            if i >= 2:
                aev[i - 2][0].record()
            lpk.lpk_kahan_sgd_step(dev.lists[0], dev.fl_theta, dev.fl_next, dev.fl_grad, cfg.lr_q16(args.warmup), cfg.wd_q16,
                                   dev.vmax, dev.status)
            if i >= 2:
                aev[i - 2][1].record()
        torch.cuda.synchronize()
        all_stores = {"ms": sum(e[0].elapsed_time(e[1]) for e in aev) / K}
        for L in dev.lists:
            lpk.lpk_tensor_list_set_option(L, lpk.LPK_OPT_STORE_ALL, 0)

    # the same whole step replayed from HIP graphs (one recording per resident gradient draw): what launch
    # overhead is left once the three calls are captured -- matters for the small, launch-bound workloads
    graph = None
    if mu_q16 is None and not args.adam and not cfg.reselect:
        graphs = [dev.capture_step(args.warmup, k) for k in range(n_src)]
        for k in range(n_src):
            graphs[k].replay()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for i in range(K):
            graphs[i % n_src].replay()
        torch.cuda.synchronize()
        gwall = time.perf_counter() - t2
        graph = {"ms_per_step": gwall * 1e3 / K, "value": cfg.n_params / (gwall / K) / 1e9, "unit": "Gparam/s"}
        del graphs
        graphs = [dev.capture_step(args.warmup, k, fused=True) for k in range(n_src)]
        for k in range(n_src):
            graphs[k].replay()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for i in range(K):
            graphs[i % n_src].replay()
        torch.cuda.synchronize()
        gwall = time.perf_counter() - t2
        graph["fused_ms_per_step"] = gwall * 1e3 / K
        graph["fused_value"] = cfg.n_params / (gwall / K) / 1e9
        del graphs

    sel_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / K
    qnt_ms = sum(e[1].elapsed_time(e[2]) for e in ev) / K
    upd_ms = sum(e[2].elapsed_time(e[3]) for e in ev) / K
    ms_per_step = wall * 1e3 / K
    status = int(dev.status.cpu().numpy().view("uint32")[0])

    copy = mix = None
    if args.copy_gib > 0:
        nb = int(args.copy_gib * (1 << 30)) // 16 * 16
        a = torch.empty(nb, dtype=torch.uint8, device="cuda:0")
        b = torch.zeros(nb, dtype=torch.uint8, device="cuda:0")
        lpk.lpk_stream_copy(a, b, nb)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 10
        e0.record()
        for _ in range(reps):
            lpk.lpk_stream_copy(a, b, nb)
        e1.record()
        torch.cuda.synchronize()
        cms = e0.elapsed_time(e1) / reps
        copy = {"bytes_read": nb, "bytes_written": nb, "ms": cms, "GB/s": 2 * nb / (cms * 1e-3) / 1e9}
        del a, b
        # the update's own byte mix (4 read : 2 written, in place) with no arithmetic, at the headline size
        nm = min(cfg.n_params, 1 << 30) // 4096 * 4096
        a = torch.zeros(nm, dtype=torch.uint8, device="cuda:0")
        b = torch.zeros(nm, dtype=torch.uint8, device="cuda:0")
        c = torch.zeros(2 * nm, dtype=torch.uint8, device="cuda:0")
        lpk.lpk_stream_mix(a, b, c, nm)
        e0.record()
        for _ in range(reps):
            lpk.lpk_stream_mix(a, b, c, nm)
        e1.record()
        torch.cuda.synchronize()
        mms = e0.elapsed_time(e1) / reps
        mix = {"bytes_read": 4 * nm, "bytes_written": 2 * nm, "ms": mms, "GB/s": 6 * nm / (mms * 1e-3) / 1e9}
        del a, b, c

    upd_bytes = sum(n * (2 * (b // 8) + 2 * (cb // 8) + args.grad_bits // 8) for n, b, cb in zip(cfg.sizes, cfg.bits, dev.comp_bits))
    upd_bytes += 2 * (args.momentum_bits // 8) * cfg.n_params if args.momentum_bits else 0
    upd_bytes += 8 * cfg.n_params if args.adam else 0
    upd_kernel = "adam_step_kernel" if args.adam else ("momentum_step_kernel" if args.momentum_bits else "kahan_step_kernel")
    achieved = upd_bytes / (upd_ms * 1e-3) / 1e9
    traffic = traffic_all = None
    tpath = os.path.join(ROOT, "profiles", "traffic_config%d.json" % cfg.id)
    if os.path.exists(tpath) and not args.lr_q16 and args.grad_bits == 16 and not args.comp_bits:
        try:
            tj = json.load(open(tpath))
            traffic = tj.get(upd_kernel + "_bytes_per_launch")
            traffic_all = tj.get(upd_kernel + "_all_stores_bytes_per_launch")
        except Exception:
            traffic = None
    if all_stores:
        a_gbs = upd_bytes / (all_stores["ms"] * 1e-3) / 1e9
        all_stores = {"bound": "hbm", "kernel": upd_kernel + " with LPK_OPT_STORE_ALL", "achieved": a_gbs, "peak": HBM_PEAK_GBS,
                      "unit": "GB/s", "frac": a_gbs / HBM_PEAK_GBS, "traffic": traffic_all, "bytes_per_launch": upd_bytes,
                      "ms": all_stores["ms"]}

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
                                                    if args.momentum_bits else "") + (", ADAM with int16 moments" if args.adam else "") + (", int%d accumulator" % args.comp_bits if args.comp_bits else "") + (", int8 gradients" if args.grad_bits == 8 else ""),
                   "n_tensors": cfg.n_tensors,
                   "n_params": cfg.n_params, "lr_q16": cfg.lr_q16(0), "wd_q16": cfg.wd_q16,
                   "grad_draws_cycled": n_src},
        "update_only": {"value": cfg.n_params / (upd_ms * 1e-3) / 1e9, "unit": "Gparam/s", "ms": upd_ms},
        "stage_ms": {"select_fraclen": sel_ms, "quantize": qnt_ms, "kahan_sgd_step": upd_ms},
        "roofline": {"bound": "hbm", "kernel": upd_kernel, "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "traffic_GB/s": (traffic / (upd_ms * 1e-3) / 1e9) if traffic else None,
                     "bytes_per_launch": upd_bytes,
                     "stores": (None if (args.adam or args.momentum_bits) else
                                "16-byte groups of theta / comp that the step leaves unchanged are not written back "
                                "(the lazy update's usual case), so the HBM traffic per launch (`traffic`) is below the "
                                "algorithmic bytes `achieved` is computed from; `roofline_all_stores` times the same kernel "
                                "writing everything"),
                     "note": ("the ADAM kernel sits where two bounds meet: its exact fp64 arithmetic (77 VALU instructions per "
                              "parameter, about 2.4 ms of issue time) and its in-place byte mix (8 read : 6 written per "
                              "parameter, 2.6-3.0 ms for the memory system alone, depending on the launch shape)") if args.adam else None},
        "roofline_all_stores": all_stores,
        "other_kernels": {
            "maxabs_f32_kernel": {"GB/s": 4 * cfg.n_params / (sel_ms * 1e-3) / 1e9, "bytes_per_launch": 4 * cfg.n_params},
            "quantize_kernel": {"GB/s": 6 * cfg.n_params / (qnt_ms * 1e-3) / 1e9, "bytes_per_launch": 6 * cfg.n_params}},
        "fused_path": fused,
        "graph_replay": graph,
        "stream_copy_yardstick": copy,
        "stream_mix_yardstick": mix,
        "device_status_word": status,
    }
    dev.close()
    del dev
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a bounded sample ...")
        cores = max(1, min(16, len(os.sched_getaffinity(0))))
        out["cpu_baseline"] = cpu_baseline(cfg, args.cpu_sample, cores, args.grad_bits)
        out["cpu_baseline_one_thread"] = cpu_baseline(cfg, args.cpu_sample // 4, 1, args.grad_bits)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()

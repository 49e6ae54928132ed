"""Host-side mirror of one training step, run through the CPU oracle.

The same order of operations as the device harness, on numpy arrays: fp32
gradients -> max-abs fraclen -> int16 gradients -> lazy update -> (optionally)
fraclen re-selection from vmax with a one-step lag.
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from oracle import ref

DT = {8: np.int8, 16: np.int16}
THREADS = max(1, min(16, len(os.sched_getaffinity(0))))


_POOL = None


def draw_grads(cfg, step, views):
    """The fp32 gradients of every tensor at `step`, drawn into `views` (independent per-tensor draws, spread over
    host threads)."""
    global _POOL
    if cfg.n_tensors < 4:
        return [cfg.grad(t, step, out=views[t]) for t in range(cfg.n_tensors)]
    if _POOL is None:
        _POOL = ThreadPoolExecutor(max_workers=THREADS)
    return list(_POOL.map(lambda t: cfg.grad(t, step, out=views[t]), range(cfg.n_tensors)))


class OracleState:
    def __init__(self, cfg, kahan=True, comp_bits=None, mom_bits=None, fl_mom0=16, sec_bits=None, fl_sec0=40, grad_bits=16):
        self.cfg, self.kahan = cfg, kahan
        nt = cfg.n_tensors
        self.comp_bits = list(comp_bits) if comp_bits is not None else list(cfg.bits)
        self.theta = [np.zeros(n, dtype=DT[b]) for n, b in zip(cfg.sizes, cfg.bits)]
        self.comp = [np.zeros(n, dtype=DT[b]) if kahan else None for n, b in zip(cfg.sizes, self.comp_bits)]
        self.grad_bits = grad_bits
        self.grad = [np.zeros(n, dtype=DT[grad_bits]) for n in cfg.sizes]
        self.d = [(b - 1) if kahan else 0 for b in self.comp_bits]
        self.fl_theta = [b - 1 for b in cfg.bits]
        self.fl_next = list(self.fl_theta)
        self.fl_grad = [grad_bits - 1] * nt
        self.vmax = [0] * nt
        self.status = ref.new_status()
        self.mom_bits = list(mom_bits) if mom_bits is not None else None
        if self.mom_bits:
            self.mom = [np.zeros(n, dtype=DT[b]) for n, b in zip(cfg.sizes, self.mom_bits)]
        self.fl_mom = [fl_mom0] * nt
        self.fl_mom_next = [fl_mom0] * nt
        self.mmax = [0] * nt
        self.sec_bits = list(sec_bits) if sec_bits is not None else None
        if self.sec_bits:
            self.sec = [np.zeros(n, dtype=DT[b]) for n, b in zip(cfg.sizes, self.sec_bits)]
        self.fl_sec = [fl_sec0] * nt
        self.fl_sec_next = [fl_sec0] * nt
        self.umax = [0] * nt

    def init_theta(self, theta0):
        def one(t):
            st = ref.new_status()
            self.fl_theta[t] = ref.select_fraclen_f32_mt(theta0[t], self.cfg.bits[t], self.fl_theta[t], st, threads=THREADS)
            ref.quantize_mt(theta0[t], self.cfg.bits[t], self.fl_theta[t], st, out=self.theta[t], threads=THREADS)
            return int(st[0])

        nt = self.cfg.n_tensors
        if nt >= 4:
            with ThreadPoolExecutor(max_workers=THREADS) as ex:
                bits = list(ex.map(one, range(nt)))
        else:
            bits = [one(t) for t in range(nt)]
        for b in bits:
            self.status[0] |= b
        self.fl_next = list(self.fl_theta)

    def quantize_grads(self, grads):
        for t, g in enumerate(grads):
            self._quantize_grad(t, g, self.status)

    def _quantize_grad(self, t, g, status):
        self.fl_grad[t] = ref.select_fraclen_f32_mt(g, self.grad_bits, self.fl_grad[t], status, threads=THREADS)
        ref.quantize_mt(g, self.grad_bits, self.fl_grad[t], status, out=self.grad[t], threads=THREADS)

    def _reselect_theta(self, t, status):
        """Fraclen of theta for the step after next: from this step's vmax (one-step lag) where the workload asks."""
        if self.cfg.reselect:
            return ref.select_fraclen_vmax(self.vmax[t], self.fl_theta[t] + self.d[t], self.cfg.bits[t],
                                           self.fl_next[t], status)
        return self.fl_next[t]

    def _update_tensor(self, t, status, lr_q16, wd_q16):
        self.vmax[t] = ref.kahan_sgd_step_mt(self.theta[t], self.comp[t], self.grad[t], self.d[t],
                                             self.fl_theta[t], self.fl_next[t], self.fl_grad[t],
                                             lr_q16, wd_q16, status, threads=THREADS)
        return (self._reselect_theta(t, status),)

    def _update_momentum_tensor(self, t, status, lr_q16, mu_q16, wd_q16):
        self.vmax[t], self.mmax[t] = ref.momentum_sgd_step_mt(
            self.theta[t], self.comp[t], self.mom[t], self.grad[t], self.d[t], self.fl_theta[t], self.fl_next[t],
            self.fl_mom[t], self.fl_mom_next[t], self.fl_grad[t], lr_q16, mu_q16, wd_q16, status, threads=THREADS)
        return (self._reselect_theta(t, status),
                ref.select_fraclen_vmax(self.mmax[t], self.fl_mom_next[t], self.mom_bits[t], self.fl_mom_next[t], status))

    def _update_adam_tensor(self, t, status, *hyper):
        self.vmax[t], self.mmax[t], self.umax[t] = ref.adam_step_mt(
            self.theta[t], self.comp[t], self.mom[t], self.sec[t], self.grad[t], self.d[t], self.fl_theta[t], self.fl_next[t],
            self.fl_mom[t], self.fl_mom_next[t], self.fl_sec[t], self.fl_sec_next[t], self.fl_grad[t], *hyper,
            status=status, threads=THREADS)
        return (self._reselect_theta(t, status),
                ref.select_fraclen_vmax(self.mmax[t], self.fl_mom_next[t], self.mom_bits[t], self.fl_mom_next[t], status),
                ref.select_fraclen_vmax(self.umax[t], self.fl_sec_next[t], self.sec_bits[t], self.fl_sec_next[t], status))

    def _over_tensors(self, update_tensor, args, grads=None):
        """Run `update_tensor(t, status, *args)` (after quantizing grads[t], when gradients are given) for every
        tensor and rotate the fraclen lists it returns.  Tensors are independent, so lists of four or more are spread
        over host threads, each worker collecting its status bits in a word of its own (OR-ed together at the end):
        the same calls with the same results as the serial order.  Large tensors still split their element range
        inside the *_mt routines."""
        nt = self.cfg.n_tensors
        nexts = [None] * nt

        def one(t):
            st = ref.new_status()
            if grads is not None:
                self._quantize_grad(t, grads[t], st)
            nexts[t] = update_tensor(t, st, *args)
            return int(st[0])

        if nt >= 4:
            order = sorted(range(nt), key=lambda t: -self.cfg.sizes[t])
            with ThreadPoolExecutor(max_workers=THREADS) as ex:
                bits = list(ex.map(one, order))
        else:
            bits = [one(t) for t in range(nt)]
        for b in bits:
            self.status[0] |= b
        self.fl_theta, self.fl_next = self.fl_next, [n[0] for n in nexts]
        if len(nexts[0]) > 1:
            self.fl_mom, self.fl_mom_next = self.fl_mom_next, [n[1] for n in nexts]
        if len(nexts[0]) > 2:
            self.fl_sec, self.fl_sec_next = self.fl_sec_next, [n[2] for n in nexts]

    def update(self, lr_q16, wd_q16=0, grads=None):
        self._over_tensors(self._update_tensor, (lr_q16, wd_q16), grads)

    def update_momentum(self, lr_q16, mu_q16, wd_q16=0, grads=None):
        self._over_tensors(self._update_momentum_tensor, (lr_q16, mu_q16, wd_q16), grads)

    def update_adam(self, hyper, grads=None):
        """hyper = (lr_q16, lr_exp, beta1_q16, beta2_q16, eps_q16, eps_exp)."""
        self._over_tensors(self._update_adam_tensor, tuple(hyper), grads)

    def step(self, step_idx, grads, mu_q16=None):
        """One whole-path step: per tensor, gradient fraclen selection and quantization, then the update."""
        if mu_q16 is None:
            self.update(self.cfg.lr_q16(step_idx), self.cfg.wd_q16, grads)
        else:
            self.update_momentum(self.cfg.lr_q16(step_idx), mu_q16, self.cfg.wd_q16, grads)

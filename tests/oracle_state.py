"""Host-side mirror of one training step, run through the CPU oracle.

The same order of operations as the device harness, on numpy arrays: fp32
gradients -> max-abs fraclen -> int16 gradients -> lazy update -> (optionally)
fraclen re-selection from vmax with a one-step lag.
"""
import os

import numpy as np

from oracle import ref

DT = {8: np.int8, 16: np.int16}
THREADS = max(1, min(16, len(os.sched_getaffinity(0))))


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
        for t, x in enumerate(theta0):
            self.fl_theta[t] = ref.select_fraclen_f32(x, self.cfg.bits[t], self.fl_theta[t], self.status)
            ref.quantize_mt(x, self.cfg.bits[t], self.fl_theta[t], self.status, out=self.theta[t], threads=THREADS)
        self.fl_next = list(self.fl_theta)

    def quantize_grads(self, grads):
        for t, g in enumerate(grads):
            self.fl_grad[t] = ref.select_fraclen_f32(g, self.grad_bits, self.fl_grad[t], self.status)
            ref.quantize_mt(g, self.grad_bits, self.fl_grad[t], self.status, out=self.grad[t], threads=THREADS)

    def update(self, lr_q16, wd_q16=0):
        new_next = list(self.fl_next)
        for t in range(self.cfg.n_tensors):
            self.vmax[t] = ref.kahan_sgd_step_mt(self.theta[t], self.comp[t], self.grad[t], self.d[t],
                                                 self.fl_theta[t], self.fl_next[t], self.fl_grad[t],
                                                 lr_q16, wd_q16, self.status, threads=THREADS)
            if self.cfg.reselect:
                new_next[t] = ref.select_fraclen_vmax(self.vmax[t], self.fl_theta[t] + self.d[t], self.cfg.bits[t],
                                                      self.fl_next[t], self.status)
        self.fl_theta, self.fl_next = self.fl_next, new_next

    def update_momentum(self, lr_q16, mu_q16, wd_q16=0):
        new_next, new_mnext = list(self.fl_next), list(self.fl_mom_next)
        for t in range(self.cfg.n_tensors):
            self.vmax[t], self.mmax[t] = ref.momentum_sgd_step_mt(
                self.theta[t], self.comp[t], self.mom[t], self.grad[t], self.d[t], self.fl_theta[t], self.fl_next[t],
                self.fl_mom[t], self.fl_mom_next[t], self.fl_grad[t], lr_q16, mu_q16, wd_q16, self.status, threads=THREADS)
            if self.cfg.reselect:
                new_next[t] = ref.select_fraclen_vmax(self.vmax[t], self.fl_theta[t] + self.d[t], self.cfg.bits[t],
                                                      self.fl_next[t], self.status)
            new_mnext[t] = ref.select_fraclen_vmax(self.mmax[t], self.fl_mom_next[t], self.mom_bits[t],
                                                   self.fl_mom_next[t], self.status)
        self.fl_theta, self.fl_next = self.fl_next, new_next
        self.fl_mom, self.fl_mom_next = self.fl_mom_next, new_mnext

    def update_adam(self, hyper):
        """hyper = (lr_q16, lr_exp, beta1_q16, beta2_q16, eps_q16, eps_exp)."""
        new_next, new_mnext, new_unext = list(self.fl_next), list(self.fl_mom_next), list(self.fl_sec_next)
        for t in range(self.cfg.n_tensors):
            self.vmax[t], self.mmax[t], self.umax[t] = ref.adam_step_mt(
                self.theta[t], self.comp[t], self.mom[t], self.sec[t], self.grad[t], self.d[t], self.fl_theta[t], self.fl_next[t],
                self.fl_mom[t], self.fl_mom_next[t], self.fl_sec[t], self.fl_sec_next[t], self.fl_grad[t], *hyper,
                status=self.status, threads=THREADS)
            if self.cfg.reselect:
                new_next[t] = ref.select_fraclen_vmax(self.vmax[t], self.fl_theta[t] + self.d[t], self.cfg.bits[t],
                                                      self.fl_next[t], self.status)
            new_mnext[t] = ref.select_fraclen_vmax(self.mmax[t], self.fl_mom_next[t], self.mom_bits[t],
                                                   self.fl_mom_next[t], self.status)
            new_unext[t] = ref.select_fraclen_vmax(self.umax[t], self.fl_sec_next[t], self.sec_bits[t],
                                                   self.fl_sec_next[t], self.status)
        self.fl_theta, self.fl_next = self.fl_next, new_next
        self.fl_mom, self.fl_mom_next = self.fl_mom_next, new_mnext
        self.fl_sec, self.fl_sec_next = self.fl_sec_next, new_unext

    def step(self, step_idx, grads, mu_q16=None):
        self.quantize_grads(grads)
        if mu_q16 is None:
            self.update(self.cfg.lr_q16(step_idx), self.cfg.wd_q16)
        else:
            self.update_momentum(self.cfg.lr_q16(step_idx), mu_q16, self.cfg.wd_q16)

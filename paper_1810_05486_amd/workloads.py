"""Seeded synthetic workloads: parameter-set shapes and fp32 input draws.

This module holds NONE of the method's arithmetic -- no quantization, no
fraclen rule, no update.  It only says which tensors a configuration has and
draws their fp32 initial values and fp32 gradients from a counter-based
generator (numpy's Philox keyed by (seed, config, tensor, step, role, chunk)),
so the GPU harness and the CPU-oracle harness get byte-identical inputs and any
chunk can be regenerated on its own.

The five configurations stand in for the paper's trained networks (Section 4:
LeNet/MNIST, ResNet/ImageNet-class models): only the SHAPES of the parameter
sets and the value distributions of the gradients matter to the update path.
Learning rates are the Q0.16 integers RNE(lr * 2^16) of the decimal literals.
"""
import math
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

CHUNK = 1 << 22            # elements per independently keyed draw
ROLE_THETA0, ROLE_GRAD, ROLE_SIGMA = 1, 2, 3


def _rng(seed, config, tensor, step, role, chunk):
    key = np.array([(seed << 8) | config, (tensor << 36) | (step << 16) | (role << 12) | chunk], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def _host_threads():
    return max(1, min(16, len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else os.cpu_count() or 1))


def _draw(n, fill, seed, config, tensor, step, role, out=None):
    """fill(rng, m) -> float32[m]; chunks are independent, so large tensors are drawn on a thread pool."""
    if out is None:
        out = np.empty(n, dtype=np.float32)
    if n <= CHUNK:
        out[:] = fill(_rng(seed, config, tensor, step, role, 0), n)
        return out

    def work(ci):
        lo = ci * CHUNK
        hi = min(n, lo + CHUNK)
        out[lo:hi] = fill(_rng(seed, config, tensor, step, role, ci), hi - lo)

    with ThreadPoolExecutor(max_workers=_host_threads()) as ex:
        list(ex.map(work, range((n + CHUNK - 1) // CHUNK)))
    return out


# ---- parameter-set shapes ------------------------------------------------------------------------------

def lenet5_shapes():
    return [(20, 1, 5, 5), (20,), (50, 20, 5, 5), (50,), (500, 800), (500,), (10, 500), (10,)]


def _bn(c):
    return [(c,), (c,)]


def resnet18_shapes():
    s = [(64, 3, 7, 7)] + _bn(64)
    cin = 64
    for stage, w in enumerate((64, 128, 256, 512)):
        for block in range(2):
            s += [(w, cin if block == 0 else w, 3, 3)] + _bn(w) + [(w, w, 3, 3)] + _bn(w)
            if block == 0 and stage > 0:
                s += [(w, cin, 1, 1)] + _bn(w)
        cin = w
    return s + [(1000, 512), (1000,)]


def resnet50_shapes():
    s = [(64, 3, 7, 7)] + _bn(64)
    cin = 64
    for w, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for block in range(blocks):
            s += [(w, cin, 1, 1)] + _bn(w) + [(w, w, 3, 3)] + _bn(w) + [(4 * w, w, 1, 1)] + _bn(4 * w)
            if block == 0:
                s += [(4 * w, cin, 1, 1)] + _bn(4 * w)
            cin = 4 * w
    return s + [(1000, 2048), (1000,)]


def _numel(shape):
    return int(np.prod(shape, dtype=np.int64))


def _fan_in(shape):
    return _numel(shape[1:]) if len(shape) >= 2 else 1


class Config:
    """One synthetic workload.  bits[t] is the width of theta AND comp of tensor t; grads are int16."""

    def __init__(self, cid, name, shapes, bits, steps, lr_schedule, wd_q16, grad_kind, reselect, seed=0,
                 grad_cycle=None):
        self.id, self.name, self.shapes, self.bits = cid, name, shapes, bits
        self.steps, self.lr_schedule, self.wd_q16 = steps, lr_schedule, wd_q16
        self.grad_kind, self.reselect, self.seed, self.grad_cycle = grad_kind, reselect, seed, grad_cycle
        self.sizes = [_numel(s) for s in shapes]
        self.n_tensors = len(shapes)
        self.n_params = sum(self.sizes)

    # -- scalars ------------------------------------------------------------------------------------
    def lr_q16(self, step):
        """Q0.16 learning rate at a 0-based step index."""
        q = self.lr_schedule[0][1]
        for start, val in self.lr_schedule:
            if step >= start:
                q = val
        return q

    def bytes_per_step(self):
        """Algorithmic HBM bytes of one update: theta and comp read + written, int16 grad read."""
        return sum(n * (4 * b // 8 + 2) for n, b in zip(self.sizes, self.bits))

    # -- draws ----------------------------------------------------------------------------------------
    def _count(self, t, count):
        n = self.sizes[t]
        if count is None or count >= n:
            return n
        assert count % CHUNK == 0, "a prefix draw ends on a chunk boundary"
        return count

    def theta0(self, t, out=None, count=None):
        """fp32 initial parameters of tensor t (count: only its first `count` elements, same values)."""
        shape = self.shapes[t]
        if self.id in (1, 5):
            b = 0.5
        else:
            b = _fan_in(shape) ** -0.5 if len(shape) >= 2 else 0.5
        fill = lambda rng, m: ((2.0 * rng.random(m) - 1.0) * b).astype(np.float32)
        return _draw(self._count(t, count), fill, self.seed, self.id, t, 0, ROLE_THETA0, out)

    def grad_scale(self, t):
        kind = self.grad_kind
        if kind == "normal_1e-3":
            return 1e-3
        if kind == "normal_loguniform":           # std drawn once per tensor, log-uniform in [1e-5, 1e-2]
            u = _rng(self.seed, self.id, t, 0, ROLE_SIGMA, 0).random()
            return float(10.0 ** (-5.0 + 3.0 * u))
        if kind == "laplace_1e-4":
            return 1e-4
        if kind == "normal_fanin":                # std = 1e-4 * fan_in^-1/2
            return 1e-4 * _fan_in(self.shapes[t]) ** -0.5
        raise ValueError(kind)

    def grad(self, t, step, out=None, count=None):
        """fp32 gradient of tensor t at a 0-based step (a fresh draw per step, or a cycle of grad_cycle draws);
        count: only its first `count` elements, same values."""
        key_step = step % self.grad_cycle if self.grad_cycle else step
        scale = self.grad_scale(t)
        if self.grad_kind == "laplace_1e-4":
            fill = lambda rng, m: rng.laplace(0.0, scale, m).astype(np.float32)
        else:
            sc = np.float32(scale)
            fill = lambda rng, m: rng.standard_normal(m, dtype=np.float32) * sc
        return _draw(self._count(t, count), fill, self.seed, self.id, t, key_step, ROLE_GRAD, out)


def config(cid, big_elems=1 << 30, n_tiny=10000):
    """The five workloads.  `big_elems` / `n_tiny` shrink config 5 for quick checks (full size by default)."""
    if cid == 1:
        return Config(1, "single int8 tensor, 65536 elements", [(65536,)], [8], 100, [(0, 655)], 0,
                      "normal_1e-3", False)
    if cid == 2:
        sh = lenet5_shapes()
        return Config(2, "LeNet-5-shaped set, int16, fraclen re-selected every step", sh, [16] * len(sh), 1000,
                      [(0, 3277)], 0, "normal_loguniform", True)
    if cid == 3:
        sh = resnet18_shapes()
        return Config(3, "ResNet-18-shaped set, int8, stepped lr", sh, [8] * len(sh), 1000,
                      [(0, 6554), (300, 655), (600, 66)], 0, "laplace_1e-4", False)
    if cid == 4:
        sh = resnet50_shapes()
        bits = [8] * (len(sh) - 2) + [16, 16]     # classifier weight and bias in 16 bits (Section 3 guideline)
        return Config(4, "ResNet-50-shaped set, int8 with int16 classifier, weight decay", sh, bits, 200,
                      [(0, 6554)], 7, "normal_fanin", False)
    if cid == 5:
        sh = [(big_elems,)] + [(256,)] * n_tiny
        return Config(5, "stress: one %d-element int8 tensor + %d tensors of 256" % (big_elems, n_tiny), sh,
                      [8] * len(sh), 50, [(0, 655)], 0, "normal_1e-3", False, grad_cycle=3)
    raise ValueError("config id must be 1..5")


def q16_pair(x):
    """A positive real as a 16-bit mantissa and an exponent: x ~ q * 2^-(16 + e), 0 <= e <= 48, the largest e that
    keeps q within 16 bits (host-side scalar conversion, like the Q0.16 learning rates above)."""
    if x <= 0.0:
        return 0, 0
    e = 0
    while e < 48 and x * 2.0 ** (16 + e + 1) <= 65535.0:
        e += 1
    return min(65535, int(round(x * 2.0 ** (16 + e)))), e


def adam_hyper(step, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8):
    """(lr_q16, lr_exp, beta1_q16, beta2_q16, eps_q16, eps_exp) for the 0-based `step`: the betas as Q0.16, the
    bias corrections 1 - beta^t (t = step + 1, with the quantized betas) folded into the step size."""
    b1_q, b2_q = int(round(beta1 * 65536)), int(round(beta2 * 65536))
    t = step + 1
    lr_t = lr * (1.0 - (b2_q / 65536.0) ** t) ** 0.5 / (1.0 - (b1_q / 65536.0) ** t)
    return q16_pair(lr_t) + (b1_q, b2_q) + q16_pair(eps)

"""ctypes front end of the CPU oracle (oracle/lpk_ref.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The GPU package never imports this module and
this module never imports the GPU package.

All functions take numpy arrays (host memory) and work in place where the C
routine does.  `status` is a one-element uint32 array that collects the
data-dependent condition bits (1 = non-finite fp32 seen, 2 = fraclen outside
the domain, tensor untouched).
"""
import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lpk_ref.c")
_LIB = os.path.join(_HERE, "liblpk_ref.so")

STATUS_NONFINITE = 1
STATUS_DOMAIN = 2


def build(force=False):
    """Compile the oracle with gcc -O2 (no vector intrinsics, no tuning flags)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-Wall", "-Wextra", "-shared", "-fPIC",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def load(path):
    """Open a built oracle library and declare its four entry points."""
    L = ctypes.CDLL(path)
    vp, u64, i32, u32, ci = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int32, ctypes.c_uint32, ctypes.c_int
    L.lpk_ref_select_fraclen_f32.argtypes = [vp, u64, ci, i32, vp, vp]
    L.lpk_ref_select_fraclen_vmax.argtypes = [u64, i32, ci, i32, vp, vp]
    L.lpk_ref_quantize.argtypes = [vp, u64, ci, i32, vp, vp]
    L.lpk_ref_kahan_sgd_step.argtypes = [vp, vp, vp, u64, ci, ci, ci, ci, i32, i32, i32, u32, u32, vp, vp]
    L.lpk_ref_momentum_sgd_step.argtypes = [vp, vp, vp, vp, u64, ci, ci, ci, ci, ci, i32, i32, i32, i32, i32,
                                            u32, u32, u32, vp, vp, vp]
    L.lpk_ref_momentum_sgd_step.restype = ci
    L.lpk_ref_adam_step.argtypes = [vp, vp, vp, vp, vp, u64, ci, ci, ci, ci, ci, ci, i32, i32, i32, i32, i32, i32, i32,
                                    u32, u32, u32, u32, u32, u32, vp, vp, vp, vp]
    L.lpk_ref_adam_step.restype = ci
    L.lpk_ref_classifier_min_bits.argtypes = [u32, u32]
    L.lpk_ref_classifier_min_bits.restype = ci
    for f in (L.lpk_ref_select_fraclen_f32, L.lpk_ref_select_fraclen_vmax,
              L.lpk_ref_quantize, L.lpk_ref_kahan_sgd_step):
        f.restype = ci
    return L


def lib():
    global _lib
    if _lib is None:
        _lib = load(build())
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data


def _bits(a):
    if a.dtype == np.int8:
        return 8
    if a.dtype == np.int16:
        return 16
    raise TypeError("DFX arrays are int8 or int16, got %s" % a.dtype)


def _check(rc):
    if rc != 0:
        raise ValueError("oracle rejected its arguments (rc=%d)" % rc)


def new_status():
    return np.zeros(1, dtype=np.uint32)


def select_fraclen_f32(x, bits, fl_default, status=None):
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.zeros(1, dtype=np.int32)
    _check(lib().lpk_ref_select_fraclen_f32(_ptr(x), x.size, bits, int(fl_default), _ptr(out), _ptr(status)))
    return int(out[0])


def select_fraclen_f32_mt(x, bits, fl_default, status=None, threads=1, chunk=1 << 22):
    """Same result as select_fraclen_f32, the scan cut into contiguous chunks on a thread pool.  The rule's result
    never grows with the maximum, so the fraclen of the whole tensor is the smallest of the chunks' fraclens; an
    all-zero chunk reports a sentinel above the rule's range and is left out (all chunks zero: fl_default).  A
    non-finite value gives the rule's lowest result in its chunk and so in the minimum.  Harness convenience for
    large tensors; the arithmetic is the single C routine."""
    x = np.ascontiguousarray(x, dtype=np.float32).reshape(-1)
    n = x.size
    if threads <= 1 or n <= chunk:
        return select_fraclen_f32(x, bits, fl_default, status)
    sentinel = 1000
    stats = []

    def work(lo):
        st = new_status()
        stats.append(st)
        return select_fraclen_f32(x[lo:min(lo + chunk, n)], bits, sentinel, st)

    with ThreadPoolExecutor(max_workers=threads) as ex:
        fls = [f for f in ex.map(work, range(0, n, chunk)) if f != sentinel]
    if status is not None:
        for st in stats:
            status[0] |= st[0]
    return min(fls) if fls else int(fl_default)


def select_fraclen_vmax(vmax, vmax_fl, bits, fl_default, status=None):
    out = np.zeros(1, dtype=np.int32)
    _check(lib().lpk_ref_select_fraclen_vmax(int(vmax), int(vmax_fl), bits, int(fl_default), _ptr(out), _ptr(status)))
    return int(out[0])


def quantize(x, bits, fl, status=None, out=None):
    x = np.ascontiguousarray(x, dtype=np.float32)
    if out is None:
        out = np.zeros(x.shape, dtype=np.int8 if bits == 8 else np.int16)
    assert out.flags.c_contiguous and out.size == x.size and _bits(out) == bits
    _check(lib().lpk_ref_quantize(_ptr(x), x.size, bits, int(fl), _ptr(out), _ptr(status)))
    return out


def kahan_sgd_step(theta, comp, grad, d, fl_in, fl_out, fl_g, lr_q, wd_q=0, status=None):
    """One lazy-update step over one tensor, in place.  Returns vmax (int).

    comp=None runs plain SGD without the accumulator.  d=None takes the
    default bits(comp)-1.
    """
    for a in (theta, comp, grad):
        assert a is None or a.flags.c_contiguous
    n = theta.size
    assert grad.size == n and (comp is None or comp.size == n)
    cb = _bits(comp) if comp is not None else 8
    if d is None:
        d = cb - 1
    vmax = np.zeros(1, dtype=np.uint64)
    _check(lib().lpk_ref_kahan_sgd_step(_ptr(theta), _ptr(comp), _ptr(grad), n,
                                        _bits(theta), cb, _bits(grad), int(d),
                                        int(fl_in), int(fl_out), int(fl_g), int(lr_q), int(wd_q),
                                        _ptr(vmax), _ptr(status)))
    return int(vmax[0])


def kahan_sgd_step_mt(theta, comp, grad, d, fl_in, fl_out, fl_g, lr_q, wd_q=0, status=None, threads=1,
                      chunk=1 << 22):
    """Same result as kahan_sgd_step, the element range cut into contiguous
    chunks that run on a thread pool (elements are independent; the chunk
    maxima are combined with an integer max).  Harness convenience for large
    tensors; the arithmetic is the single C routine above."""
    n = theta.size
    if threads <= 1 or n <= chunk:
        return kahan_sgd_step(theta, comp, grad, d, fl_in, fl_out, fl_g, lr_q, wd_q, status)
    th, gr = theta.reshape(-1), grad.reshape(-1)
    co = comp.reshape(-1) if comp is not None else None
    stats = []

    def work(lo):
        hi = min(lo + chunk, n)
        st = new_status()
        stats.append(st)
        return kahan_sgd_step(th[lo:hi], None if co is None else co[lo:hi], gr[lo:hi],
                              d if d is not None else (_bits(co) - 1 if co is not None else 0),
                              fl_in, fl_out, fl_g, lr_q, wd_q, st)

    with ThreadPoolExecutor(max_workers=threads) as ex:
        vm = max(ex.map(work, range(0, n, chunk)))
    if status is not None:
        for st in stats:
            status[0] |= st[0]
    return vm


def quantize_mt(x, bits, fl, status=None, out=None, threads=1, chunk=1 << 22):
    """Same result as quantize (elementwise), contiguous chunks on a thread pool."""
    x = np.ascontiguousarray(x, dtype=np.float32).reshape(-1)
    n = x.size
    if out is None:
        out = np.zeros(n, dtype=np.int8 if bits == 8 else np.int16)
    if threads <= 1 or n <= chunk:
        return quantize(x, bits, fl, status, out)
    flat = out.reshape(-1)
    stats = []

    def work(lo):
        hi = min(lo + chunk, n)
        st = new_status()
        stats.append(st)
        quantize(x[lo:hi], bits, fl, st, flat[lo:hi])

    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(work, range(0, n, chunk)))
    if status is not None:
        for st in stats:
            status[0] |= st[0]
    return out


def classifier_min_bits(n_classes, alpha_q16=32768):
    rc = lib().lpk_ref_classifier_min_bits(int(n_classes), int(alpha_q16))
    _check(rc if rc < 0 else 0)
    return rc


def momentum_sgd_step(theta, comp, mom, grad, d, fl_in, fl_out, fl_m_in, fl_m_out, fl_g, lr_q, mu_q, wd_q=0,
                      status=None):
    """One momentum step with the lazy update inside, in place.  Returns (vmax, mmax)."""
    for a in (theta, comp, mom, grad):
        assert a is None or a.flags.c_contiguous
    n = theta.size
    assert grad.size == n and mom.size == n and (comp is None or comp.size == n)
    cb = _bits(comp) if comp is not None else 8
    if d is None:
        d = cb - 1
    vmax, mmax = np.zeros(1, dtype=np.uint64), np.zeros(1, dtype=np.uint64)
    _check(lib().lpk_ref_momentum_sgd_step(_ptr(theta), _ptr(comp), _ptr(mom), _ptr(grad), n,
                                           _bits(theta), cb, _bits(mom), _bits(grad), int(d),
                                           int(fl_in), int(fl_out), int(fl_m_in), int(fl_m_out), int(fl_g),
                                           int(lr_q), int(mu_q), int(wd_q), _ptr(vmax), _ptr(mmax), _ptr(status)))
    return int(vmax[0]), int(mmax[0])


def momentum_sgd_step_mt(theta, comp, mom, grad, d, fl_in, fl_out, fl_m_in, fl_m_out, fl_g, lr_q, mu_q, wd_q=0,
                         status=None, threads=1, chunk=1 << 22):
    """Same result as momentum_sgd_step, contiguous chunks on a thread pool (elements are independent)."""
    n = theta.size
    if threads <= 1 or n <= chunk:
        return momentum_sgd_step(theta, comp, mom, grad, d, fl_in, fl_out, fl_m_in, fl_m_out, fl_g, lr_q, mu_q, wd_q, status)
    th, gr, mo = theta.reshape(-1), grad.reshape(-1), mom.reshape(-1)
    co = comp.reshape(-1) if comp is not None else None
    dd = d if d is not None else (_bits(co) - 1 if co is not None else 0)
    stats = []

    def work(lo):
        hi = min(lo + chunk, n)
        st = new_status()
        stats.append(st)
        return momentum_sgd_step(th[lo:hi], None if co is None else co[lo:hi], mo[lo:hi], gr[lo:hi], dd,
                                 fl_in, fl_out, fl_m_in, fl_m_out, fl_g, lr_q, mu_q, wd_q, st)

    with ThreadPoolExecutor(max_workers=threads) as ex:
        res = list(ex.map(work, range(0, n, chunk)))
    if status is not None:
        for st in stats:
            status[0] |= st[0]
    return max(r[0] for r in res), max(r[1] for r in res)


def adam_step(theta, comp, mom, sec, grad, d, fl_in, fl_out, fl_m_in, fl_m_out, fl_u_in, fl_u_out, fl_g,
              lr_q, lr_exp, b1_q, b2_q, eps_q, eps_exp, status=None):
    """One ADAM step with the lazy update inside, in place.  Returns (vmax, mmax, umax)."""
    for a in (theta, comp, mom, sec, grad):
        assert a is None or a.flags.c_contiguous
    n = theta.size
    assert grad.size == n and mom.size == n and sec.size == n and (comp is None or comp.size == n)
    cb = _bits(comp) if comp is not None else 8
    if d is None:
        d = cb - 1
    vmax, mmax, umax = (np.zeros(1, dtype=np.uint64) for _ in range(3))
    _check(lib().lpk_ref_adam_step(_ptr(theta), _ptr(comp), _ptr(mom), _ptr(sec), _ptr(grad), n,
                                   _bits(theta), cb, _bits(mom), _bits(sec), _bits(grad), int(d),
                                   int(fl_in), int(fl_out), int(fl_m_in), int(fl_m_out), int(fl_u_in), int(fl_u_out), int(fl_g),
                                   int(lr_q), int(lr_exp), int(b1_q), int(b2_q), int(eps_q), int(eps_exp),
                                   _ptr(vmax), _ptr(mmax), _ptr(umax), _ptr(status)))
    return int(vmax[0]), int(mmax[0]), int(umax[0])


def adam_step_mt(theta, comp, mom, sec, grad, d, fl_in, fl_out, fl_m_in, fl_m_out, fl_u_in, fl_u_out, fl_g,
                 lr_q, lr_exp, b1_q, b2_q, eps_q, eps_exp, status=None, threads=1, chunk=1 << 22):
    """Same result as adam_step, contiguous chunks on a thread pool (elements are independent)."""
    n = theta.size
    args = (fl_in, fl_out, fl_m_in, fl_m_out, fl_u_in, fl_u_out, fl_g, lr_q, lr_exp, b1_q, b2_q, eps_q, eps_exp)
    if threads <= 1 or n <= chunk:
        return adam_step(theta, comp, mom, sec, grad, d, *args, status)
    th, gr, mo, se = theta.reshape(-1), grad.reshape(-1), mom.reshape(-1), sec.reshape(-1)
    co = comp.reshape(-1) if comp is not None else None
    dd = d if d is not None else (_bits(co) - 1 if co is not None else 0)
    stats = []

    def work(lo):
        hi = min(lo + chunk, n)
        st = new_status()
        stats.append(st)
        return adam_step(th[lo:hi], None if co is None else co[lo:hi], mo[lo:hi], se[lo:hi], gr[lo:hi], dd, *args, st)

    with ThreadPoolExecutor(max_workers=threads) as ex:
        res = list(ex.map(work, range(0, n, chunk)))
    if status is not None:
        for st in stats:
            status[0] |= st[0]
    return tuple(max(r[k] for r in res) for k in range(3))

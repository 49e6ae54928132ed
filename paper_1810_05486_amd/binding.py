"""Python binding of liblpk.so: the same names as include/lpk.h, argument
marshalling only.  Device buffers are torch tensors (or raw integer device
addresses); every step of the path runs inside the library's kernels.

There is no fallback: if the library is missing, the first call raises.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblpk.so")

LPK_OK, LPK_ERR_INVALID_ARG, LPK_ERR_UNSUPPORTED, LPK_ERR_DEVICE = 0, -1, -2, -3
LPK_I8, LPK_I16, LPK_F32, LPK_VMAX_U64 = 1, 2, 4, 8
LPK_SEL_GRAD, LPK_SEL_THETA, LPK_SEL_MOMENTUM, LPK_SEL_SECOND = 0, 1, 2, 3
LPK_STATUS_NONFINITE, LPK_STATUS_DOMAIN = 1, 2
LPK_COMP_SHIFT_DEFAULT = 0xFF
LPK_OPT_STORE_ALL = 1
LPK_OPT_STEP_BLOCKS_PER_CU, LPK_OPT_DENSE_BLOCKS_PER_CU, LPK_OPT_ADAM_BLOCKS_PER_CU = 2, 3, 4
LPK_OPT_SCAN_BLOCKS_PER_CU, LPK_OPT_QUANT_BLOCKS_PER_CU = 5, 6


class lpk_tensor_desc(ctypes.Structure):
    _fields_ = [("theta", ctypes.c_void_p), ("comp", ctypes.c_void_p), ("grad", ctypes.c_void_p),
                ("src_f32", ctypes.c_void_p), ("n", ctypes.c_uint64),
                ("theta_dtype", ctypes.c_uint8), ("comp_dtype", ctypes.c_uint8),
                ("grad_dtype", ctypes.c_uint8), ("comp_shift", ctypes.c_uint8),
                ("momentum_dtype", ctypes.c_uint8), ("second_dtype", ctypes.c_uint8), ("reserved", ctypes.c_uint8 * 2),
                ("momentum", ctypes.c_void_p), ("second", ctypes.c_void_p)]


class lpk_adam_hyper(ctypes.Structure):
    _fields_ = [("lr_q16", ctypes.c_uint32), ("lr_exp", ctypes.c_uint32), ("beta1_q16", ctypes.c_uint32),
                ("beta2_q16", ctypes.c_uint32), ("eps_q16", ctypes.c_uint32), ("eps_exp", ctypes.c_uint32)]


class LpkError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (where, lib().lpk_error_string(code).decode(), code))


_lib = None


def lib():
    """The loaded C library (loads on first use; raises if it was never built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("liblpk.so is not built (%s); run `python -m paper_1810_05486_amd.build`. "
                               "There is no CPU fallback." % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, u32, u64, ci = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_int
        L.lpk_tensor_list_create.argtypes = [ctypes.POINTER(lpk_tensor_desc), u32, ctypes.POINTER(vp)]
        L.lpk_tensor_list_destroy.argtypes = [vp]
        L.lpk_tensor_list_set_option.argtypes = [vp, ci, ci]
        L.lpk_tensor_list_set_option.restype = ci
        L.lpk_tensor_list_size.argtypes = [vp]
        L.lpk_tensor_list_size.restype = u32
        L.lpk_tensor_list_tiles.argtypes = [vp]
        L.lpk_tensor_list_tiles.restype = u64
        L.lpk_select_fraclen.argtypes = [vp, ci, ci, vp, vp, vp, vp, vp, vp]
        L.lpk_quantize_tensor.argtypes = [vp, ci, vp, vp, vp]
        L.lpk_select_quantize.argtypes = [vp, ci, vp, vp, vp, vp]
        L.lpk_select_quantize.restype = ci
        L.lpk_kahan_sgd_step.argtypes = [vp, vp, vp, vp, u32, u32, vp, vp, vp]
        L.lpk_kahan_sgd_step_f32grad.argtypes = [vp, vp, vp, vp, u32, u32, vp, vp, vp]
        L.lpk_kahan_sgd_step_f32grad.restype = ci
        L.lpk_kahan_sgd_step_noalloc.argtypes = [ctypes.POINTER(lpk_tensor_desc), u32, vp, vp, vp, u32, u32, vp, vp, vp]
        L.lpk_kahan_sgd_step_noalloc.restype = ci
        L.lpk_momentum_sgd_step.argtypes = [vp, vp, vp, vp, vp, vp, u32, u32, u32, vp, vp, vp, vp]
        L.lpk_momentum_sgd_step.restype = ci
        L.lpk_adam_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, ctypes.POINTER(lpk_adam_hyper), vp, vp, vp, vp, vp]
        L.lpk_adam_step.restype = ci
        L.lpk_momentum_sgd_step_f32grad.argtypes = L.lpk_momentum_sgd_step.argtypes
        L.lpk_momentum_sgd_step_f32grad.restype = ci
        L.lpk_adam_step_f32grad.argtypes = L.lpk_adam_step.argtypes
        L.lpk_adam_step_f32grad.restype = ci
        L.lpk_classifier_min_bits.argtypes = [u32, u32]
        L.lpk_classifier_min_bits.restype = ci
        L.lpk_error_string.argtypes = [ci]
        L.lpk_error_string.restype = ctypes.c_char_p
        L.lpk_version.restype = ci
        for f in (L.lpk_tensor_list_create, L.lpk_tensor_list_destroy, L.lpk_select_fraclen,
                  L.lpk_quantize_tensor, L.lpk_kahan_sgd_step):
            f.restype = ci
        _lib = L
    return _lib


def _addr(x):
    """Device address of a torch tensor / raw int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _dtype_code(t):
    import torch
    if t.dtype == torch.int8:
        return LPK_I8
    if t.dtype == torch.int16:
        return LPK_I16
    raise TypeError("DFX tensors are int8 or int16, got %s" % t.dtype)


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(rc, where):
    if rc != LPK_OK:
        raise LpkError(rc, where)


def make_desc(theta, comp, grad, src_f32=None, comp_shift=LPK_COMP_SHIFT_DEFAULT, momentum=None, second=None):
    """Descriptor for one tensor from torch tensors living on the GPU."""
    d = lpk_tensor_desc()
    d.theta, d.comp, d.grad, d.src_f32 = _addr(theta), _addr(comp), _addr(grad), _addr(src_f32)
    d.n = theta.numel()
    d.theta_dtype = _dtype_code(theta)
    d.comp_dtype = _dtype_code(comp) if comp is not None else LPK_I8
    d.grad_dtype = _dtype_code(grad)
    d.comp_shift = comp_shift
    d.momentum = _addr(momentum)
    d.momentum_dtype = _dtype_code(momentum) if momentum is not None else LPK_I8
    d.second = _addr(second)
    d.second_dtype = _dtype_code(second) if second is not None else LPK_I8
    return d


class TensorList:
    """Owner of an lpk_tensor_list handle (lpk_tensor_list_create / _destroy)."""

    def __init__(self, descs):
        arr = (lpk_tensor_desc * len(descs))(*descs)
        h = ctypes.c_void_p()
        _check(lib().lpk_tensor_list_create(arr, len(descs), ctypes.byref(h)), "lpk_tensor_list_create")
        self.handle = h
        self.n_tensors = len(descs)

    @property
    def n_tiles(self):
        return lib().lpk_tensor_list_tiles(self.handle)

    def destroy(self):
        if self.handle:
            rc = lib().lpk_tensor_list_destroy(self.handle)
            self.handle = None
            _check(rc, "lpk_tensor_list_destroy")

    def __del__(self):
        try:
            if getattr(self, "handle", None):
                lib().lpk_tensor_list_destroy(self.handle)
                self.handle = None
        except Exception:
            pass


def lpk_tensor_list_create(descs):
    return TensorList(descs)


def lpk_tensor_list_set_option(tl, option, value):
    _check(lib().lpk_tensor_list_set_option(tl.handle, int(option), int(value)), "lpk_tensor_list_set_option")


def lpk_tensor_list_destroy(tl):
    tl.destroy()


def lpk_select_fraclen(tl, src_kind, dst_sel, vmax, fl_theta_in, fl_default, fl_out, status=None, stream=None):
    _check(lib().lpk_select_fraclen(tl.handle, src_kind, dst_sel, _addr(vmax), _addr(fl_theta_in), _addr(fl_default),
                                    _addr(fl_out), _addr(status), _stream(stream)), "lpk_select_fraclen")


def lpk_quantize_tensor(tl, dst_sel, fl, status=None, stream=None):
    _check(lib().lpk_quantize_tensor(tl.handle, dst_sel, _addr(fl), _addr(status), _stream(stream)),
           "lpk_quantize_tensor")


def lpk_select_quantize(tl, dst_sel, fl_guess, fl_out, status=None, stream=None):
    _check(lib().lpk_select_quantize(tl.handle, dst_sel, _addr(fl_guess), _addr(fl_out), _addr(status), _stream(stream)),
           "lpk_select_quantize")


def lpk_kahan_sgd_step(tl, fl_theta_in, fl_theta_out, fl_grad, lr_q16, wd_q16=0, vmax_out=None, status=None,
                       stream=None):
    _check(lib().lpk_kahan_sgd_step(tl.handle, _addr(fl_theta_in), _addr(fl_theta_out), _addr(fl_grad),
                                    int(lr_q16), int(wd_q16), _addr(vmax_out), _addr(status), _stream(stream)),
           "lpk_kahan_sgd_step")


def lpk_kahan_sgd_step_f32grad(tl, fl_theta_in, fl_theta_out, fl_grad, lr_q16, wd_q16=0, vmax_out=None, status=None,
                               stream=None):
    _check(lib().lpk_kahan_sgd_step_f32grad(tl.handle, _addr(fl_theta_in), _addr(fl_theta_out), _addr(fl_grad),
                                            int(lr_q16), int(wd_q16), _addr(vmax_out), _addr(status), _stream(stream)),
           "lpk_kahan_sgd_step_f32grad")


def lpk_kahan_sgd_step_noalloc(descs, fl_theta_in, fl_theta_out, fl_grad, lr_q16, wd_q16=0, vmax_out=None, status=None,
                               stream=None):
    """descs: a list of lpk_tensor_desc (see make_desc), or a ctypes array of them."""
    arr = descs if isinstance(descs, ctypes.Array) else (lpk_tensor_desc * len(descs))(*descs)
    _check(lib().lpk_kahan_sgd_step_noalloc(arr, len(arr), _addr(fl_theta_in), _addr(fl_theta_out), _addr(fl_grad),
                                            int(lr_q16), int(wd_q16), _addr(vmax_out), _addr(status), _stream(stream)),
           "lpk_kahan_sgd_step_noalloc")


def lpk_momentum_sgd_step(tl, fl_theta_in, fl_theta_out, fl_mom_in, fl_mom_out, fl_grad, lr_q16, mu_q16, wd_q16=0,
                          vmax_out=None, mmax_out=None, status=None, stream=None):
    _check(lib().lpk_momentum_sgd_step(tl.handle, _addr(fl_theta_in), _addr(fl_theta_out), _addr(fl_mom_in),
                                       _addr(fl_mom_out), _addr(fl_grad), int(lr_q16), int(mu_q16), int(wd_q16),
                                       _addr(vmax_out), _addr(mmax_out), _addr(status), _stream(stream)),
           "lpk_momentum_sgd_step")


def lpk_momentum_sgd_step_f32grad(tl, fl_theta_in, fl_theta_out, fl_mom_in, fl_mom_out, fl_grad, lr_q16, mu_q16, wd_q16=0,
                                  vmax_out=None, mmax_out=None, status=None, stream=None):
    _check(lib().lpk_momentum_sgd_step_f32grad(tl.handle, _addr(fl_theta_in), _addr(fl_theta_out), _addr(fl_mom_in),
                                               _addr(fl_mom_out), _addr(fl_grad), int(lr_q16), int(mu_q16), int(wd_q16),
                                               _addr(vmax_out), _addr(mmax_out), _addr(status), _stream(stream)),
           "lpk_momentum_sgd_step_f32grad")


def lpk_adam_step(tl, fl_theta_in, fl_theta_out, fl_mom_in, fl_mom_out, fl_sec_in, fl_sec_out, fl_grad, hyper,
                  vmax_out=None, mmax_out=None, umax_out=None, status=None, stream=None):
    """hyper: an lpk_adam_hyper, or a tuple (lr_q16, lr_exp, beta1_q16, beta2_q16, eps_q16, eps_exp)."""
    h = hyper if isinstance(hyper, lpk_adam_hyper) else lpk_adam_hyper(*[int(x) for x in hyper])
    _check(lib().lpk_adam_step(tl.handle, _addr(fl_theta_in), _addr(fl_theta_out), _addr(fl_mom_in), _addr(fl_mom_out),
                               _addr(fl_sec_in), _addr(fl_sec_out), _addr(fl_grad), ctypes.byref(h),
                               _addr(vmax_out), _addr(mmax_out), _addr(umax_out), _addr(status), _stream(stream)),
           "lpk_adam_step")


def lpk_adam_step_f32grad(tl, fl_theta_in, fl_theta_out, fl_mom_in, fl_mom_out, fl_sec_in, fl_sec_out, fl_grad, hyper,
                          vmax_out=None, mmax_out=None, umax_out=None, status=None, stream=None):
    """lpk_adam_step fed from the fp32 gradients; hyper as there."""
    h = hyper if isinstance(hyper, lpk_adam_hyper) else lpk_adam_hyper(*[int(x) for x in hyper])
    _check(lib().lpk_adam_step_f32grad(tl.handle, _addr(fl_theta_in), _addr(fl_theta_out), _addr(fl_mom_in), _addr(fl_mom_out),
                                       _addr(fl_sec_in), _addr(fl_sec_out), _addr(fl_grad), ctypes.byref(h),
                                       _addr(vmax_out), _addr(mmax_out), _addr(umax_out), _addr(status), _stream(stream)),
           "lpk_adam_step_f32grad")


def lpk_classifier_min_bits(n_classes, alpha_q16=32768):
    rc = lib().lpk_classifier_min_bits(int(n_classes), int(alpha_q16))
    if rc < 0:
        raise LpkError(rc, "lpk_classifier_min_bits")
    return rc


def lpk_version():
    return lib().lpk_version()

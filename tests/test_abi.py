"""The C-ABI library loads without a GPU, exports every function the header declares, and rejects bad
arguments on the host before touching the device (no compute calls here)."""
import ctypes
import os
import re

import pytest

from paper_1810_05486_amd import binding as lpk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "lpk.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lpk_[a-z0-9_]+)\s*\(", text)))


def test_header_functions_are_exported():
    names = declared_functions()
    assert {"lpk_quantize_tensor", "lpk_select_fraclen", "lpk_kahan_sgd_step", "lpk_tensor_list_create",
            "lpk_tensor_list_destroy"} <= set(names)
    L = lpk.lib()
    for n in names:
        assert hasattr(L, n), "liblpk.so does not export %s" % n


def test_binding_has_the_same_names():
    for n in declared_functions():
        if n in ("lpk_error_string", "lpk_tensor_list_size", "lpk_tensor_list_tiles"):
            continue
        assert hasattr(lpk, n), n


def test_descriptor_layout_matches_header():
    assert ctypes.sizeof(lpk.lpk_tensor_desc) == 64 and lpk.lpk_tensor_desc.momentum.offset == 48
    assert lpk.lpk_tensor_desc.second.offset == 56 and lpk.lpk_tensor_desc.second_dtype.offset == 45
    assert ctypes.sizeof(lpk.lpk_adam_hyper) == 24
    assert lpk.lpk_tensor_desc.n.offset == 32 and lpk.lpk_tensor_desc.comp_shift.offset == 43


def test_error_strings():
    L = lpk.lib()
    assert L.lpk_error_string(0) == b"ok"
    assert L.lpk_error_string(-1) == b"invalid argument"
    assert L.lpk_error_string(-77) == b"unknown lpk status code"
    assert L.lpk_version() >= 100


def _desc(**kw):
    d = lpk.lpk_tensor_desc()
    d.theta, d.comp, d.grad, d.src_f32, d.n = 0x1000, 0x2000, 0x3000, 0x4000, 64
    d.theta_dtype, d.comp_dtype, d.grad_dtype, d.comp_shift = lpk.LPK_I8, lpk.LPK_I8, lpk.LPK_I16, 0xFF
    for k, v in kw.items():
        setattr(d, k, v)
    return d


@pytest.mark.parametrize("kw", [dict(theta_dtype=3), dict(grad_dtype=lpk.LPK_F32), dict(comp_dtype=0),
                                dict(comp_shift=25), dict(theta=None), dict(grad=None),
                                dict(grad=0x3001), dict(theta=0x1001, theta_dtype=lpk.LPK_I16),
                                dict(src_f32=0x4002)])
def test_create_rejects_bad_descriptors_on_the_host(kw):
    h = ctypes.c_void_p(123)
    arr = (lpk.lpk_tensor_desc * 1)(_desc(**kw))
    assert lpk.lib().lpk_tensor_list_create(arr, 1, ctypes.byref(h)) == lpk.LPK_ERR_INVALID_ARG
    assert h.value is None


def test_null_and_range_arguments():
    L = lpk.lib()
    h = ctypes.c_void_p()
    assert L.lpk_tensor_list_create(None, 1, ctypes.byref(h)) == lpk.LPK_ERR_INVALID_ARG
    arr = (lpk.lpk_tensor_desc * 1)(_desc())
    assert L.lpk_tensor_list_create(arr, 0, ctypes.byref(h)) == lpk.LPK_ERR_INVALID_ARG
    assert L.lpk_tensor_list_create(arr, 1, None) == lpk.LPK_ERR_INVALID_ARG
    assert L.lpk_tensor_list_destroy(None) == lpk.LPK_OK
    assert L.lpk_tensor_list_size(None) == 0 and L.lpk_tensor_list_tiles(None) == 0
    assert L.lpk_kahan_sgd_step(None, 8, 8, 8, 1, 0, None, None, None) == lpk.LPK_ERR_INVALID_ARG
    assert L.lpk_quantize_tensor(None, 0, 8, None, None) == lpk.LPK_ERR_INVALID_ARG
    assert L.lpk_select_fraclen(None, lpk.LPK_F32, 0, None, None, 8, 8, None, None) == lpk.LPK_ERR_INVALID_ARG


def test_classifier_min_bits_matches_the_oracle_everywhere_on_the_host():
    """Host-only entry point: compared with the oracle's definition-level search (no GPU involved)."""
    from oracle import ref
    for n in list(range(2, 300)) + [1000, 1001, 4097, 65536, 1 << 20, (1 << 32) - 1]:
        for a_q in (32768, 1, 2, 65535, 6554, 16384, 40000):
            assert lpk.lpk_classifier_min_bits(n, a_q) == ref.classifier_min_bits(n, a_q), (n, a_q)
    L = lpk.lib()
    assert L.lpk_classifier_min_bits(1, 32768) == lpk.LPK_ERR_INVALID_ARG
    assert L.lpk_classifier_min_bits(10, 0) == lpk.LPK_ERR_INVALID_ARG
    assert L.lpk_classifier_min_bits(10, 65536) == lpk.LPK_ERR_INVALID_ARG


def test_header_is_plain_c_and_links(tmp_path):
    """include/lpk.h compiles as C99 with warnings as errors, and a C program linked against liblpk.so calls the
    host-only entry points (no GPU needed)."""
    import subprocess
    src = tmp_path / "use_lpk.c"
    src.write_text(r'''
#include "lpk.h"
#include <stdio.h>
#include <string.h>
int main(void)
{
  lpk_tensor_desc d;
  lpk_adam_hyper h = {66u, 0u, 58982u, 65470u, 0u, 0u};
  lpk_tensor_list* list = (lpk_tensor_list*)0;
  memset(&d, 0, sizeof d);
  if (sizeof(d) != 64 || sizeof(h) != 24) return 2;
  if (lpk_version() < 100) return 3;
  if (lpk_classifier_min_bits(10u, 32768u) != 6 || lpk_classifier_min_bits(1000u, 32768u) != 12) return 4;
  if (strcmp(lpk_error_string(LPK_ERR_INVALID_ARG), "invalid argument") != 0) return 5;
  if (lpk_tensor_list_create(&d, 0u, &list) != LPK_ERR_INVALID_ARG || list) return 6;   /* rejected on the host */
  if (lpk_tensor_list_size(list) != 0u || lpk_tensor_list_destroy(list) != LPK_OK) return 7;
  if (lpk_adam_step(list, 0, 0, 0, 0, 0, 0, 0, &h, 0, 0, 0, 0, 0) != LPK_ERR_INVALID_ARG) return 8;
  if (lpk_adam_step_f32grad(list, 0, 0, 0, 0, 0, 0, 0, &h, 0, 0, 0, 0, 0) != LPK_ERR_INVALID_ARG) return 9;
  if (lpk_momentum_sgd_step_f32grad(list, 0, 0, 0, 0, 0, 655u, 58982u, 0u, 0, 0, 0, 0) != LPK_ERR_INVALID_ARG) return 10;
  if (lpk_tensor_list_set_option(list, LPK_OPT_STORE_ALL, 1) != LPK_ERR_INVALID_ARG) return 11;
  if (lpk_select_quantize(list, LPK_SEL_GRAD, 0, 0, 0, 0) != LPK_ERR_INVALID_ARG) return 12;
  puts("ok");
  return 0;
}
''')
    exe = tmp_path / "use_lpk"
    libdir = os.path.dirname(lpk.LIB_PATH)
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                           str(src), "-o", str(exe), "-L", libdir, "-llpk", "-Wl,-rpath," + libdir,
                           "-Wl,-rpath,/opt/rocm/lib", "-Wl,--allow-shlib-undefined"])
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.strip() == "ok", (r.returncode, r.stdout, r.stderr[-2000:])


def test_noalloc_step_rejects_what_does_not_fit_before_launching():
    """Limits and argument errors of lpk_kahan_sgd_step_noalloc are found on the host: nothing touches a device."""
    d = lpk.lpk_tensor_desc()
    d.theta, d.comp, d.grad, d.n = 0x1000, 0x2000, 0x3000, 256
    d.theta_dtype, d.comp_dtype, d.grad_dtype, d.comp_shift = lpk.LPK_I8, lpk.LPK_I8, lpk.LPK_I16, 0xFF
    many = (lpk.lpk_tensor_desc * 16385)(*([d] * 16385))
    assert lpk.lib().lpk_kahan_sgd_step_noalloc(many, 16385, 8, 8, 8, 1, 0, None, None, None) == lpk.LPK_ERR_UNSUPPORTED
    d.n = (1 << 31) + 1                               # 524289 tiles
    one = (lpk.lpk_tensor_desc * 1)(d)
    assert lpk.lib().lpk_kahan_sgd_step_noalloc(one, 1, 8, 8, 8, 1, 0, None, None, None) == lpk.LPK_ERR_UNSUPPORTED
    d.n = 256
    one = (lpk.lpk_tensor_desc * 1)(d)
    assert lpk.lib().lpk_kahan_sgd_step_noalloc(one, 1, 8, 8, 8, 65536, 0, None, None, None) == lpk.LPK_ERR_INVALID_ARG
    assert lpk.lib().lpk_kahan_sgd_step_noalloc(one, 1, None, 8, 8, 1, 0, None, None, None) == lpk.LPK_ERR_INVALID_ARG
    assert lpk.lib().lpk_kahan_sgd_step_noalloc(None, 1, 8, 8, 8, 1, 0, None, None, None) == lpk.LPK_ERR_INVALID_ARG
    assert lpk.lib().lpk_kahan_sgd_step_noalloc(one, 0, 8, 8, 8, 1, 0, None, None, None) == lpk.LPK_ERR_INVALID_ARG
    d.comp_shift = 25
    one = (lpk.lpk_tensor_desc * 1)(d)
    assert lpk.lib().lpk_kahan_sgd_step_noalloc(one, 1, 8, 8, 8, 1, 0, None, None, None) == lpk.LPK_ERR_INVALID_ARG

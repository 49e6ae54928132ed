"""The oracle's C source under the undefined-behaviour sanitizer (CPU only): a copy built with
-fsanitize=undefined -fno-sanitize-recover aborts on the first signed overflow, oversized shift or misaligned
access, so the brute-force cases are run through it in a child process and must come back clean."""
import os
import subprocess
import sys

from oracle import ref

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(os.path.dirname(ref.__file__), "lpk_ref.c")

CHILD = r"""
import sys
sys.path.insert(0, %(root)r); sys.path.insert(0, %(tests)r)
from oracle import ref
ref._lib = ref.load(%(so)r)
import test_oracle_bruteforce as bf, test_oracle_momentum as mom, test_oracle_adam as adam, test_oracle_pins as pins
bf.test_step_random_domain(1); bf.test_step_saturation_and_cap(); bf.test_quantize_bruteforce(16)
bf.test_fraclen_is_largest_non_saturating(16); bf.test_fraclen_from_vmax_bruteforce(8)
mom.test_momentum_step_bruteforce(1); adam.test_adam_step_bruteforce(1)
adam.test_adam_out_of_domain_and_bad_arguments(); pins.test_quantize_hand_cases(); pins.test_fraclen_hand_cases()
print("sanitized oracle: clean")
"""


def test_oracle_has_no_undefined_behaviour(tmp_path):
    so = tmp_path / "lpk_ref_ubsan.so"
    subprocess.check_call(["gcc", "-O1", "-g", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-static-libubsan",
                           "-shared", "-fPIC", "-o", str(so), SRC, "-lm"])
    code = CHILD % dict(root=ROOT, tests=os.path.join(ROOT, "tests"), so=str(so))
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0 and "sanitized oracle: clean" in r.stdout, (r.returncode, r.stdout[-2000:], r.stderr[-4000:])

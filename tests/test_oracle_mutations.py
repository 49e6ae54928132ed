"""Do the pins bite?  Plant one plausible mistake at a time in a COPY of the oracle source (on the
CPU), build it, and require that the brute-force / pin tests reject it.  A mutation that survives
means a hole in the pins."""
import os
import subprocess

import pytest

from oracle import ref
import test_oracle_bruteforce as bf
import test_oracle_pins as pins
import test_oracle_momentum as mom
import test_oracle_adam as adam
import test_oracle_readings as readings

SRC = os.path.join(os.path.dirname(ref.__file__), "lpk_ref.c")

MUTATIONS = [
    ("ties_away_from_zero", "2 * r > p ||", "2 * r >= p ||"),
    ("ties_to_odd", "(2 * r == p && (q & 1))", "(2 * r == p && !(q & 1))"),
    ("floor_of_negatives", "if (r < 0) { r += p; q -= 1; }", "if (r < 0) { r += p; }"),
    ("step_sign_in_sum", "+ c + s;", "+ c - s;"),
    ("gradient_sign", "rescale_cap(-(wide)lr_q * g,", "rescale_cap((wide)lr_q * g,"),
    ("step_grid_forgets_d", "* g, fl_g + 16 - F);", "* g, fl_g + 16 - fl_in);"),
    ("decay_dropped", "if (wd_q) s +=", "if (0) s +="),
    ("decay_grid", "* th, fl_in + 32 - F);", "* th, fl_in + 16 - F);"),
    ("residual_grid", "rescale(r, k_theta - d)", "rescale(r, k_theta)"),
    ("theta_not_saturated", "wide thn = sat(rescale(vG, k_theta), theta_bits);", "wide thn = rescale(vG, k_theta);"),
    ("comp_not_saturated", "sat(rescale(r, k_theta - d), comp_bits)", "rescale(r, k_theta - d)"),
    ("finer_grid_ignored", "const int u = delta > 0 ? delta : 0;", "const int u = 0;"),
    ("k_theta_sign", "const int k_theta = d + u - delta;", "const int k_theta = d + u + delta;"),
    ("cap_dropped", "return clampw(rescale(x, k), -CAP40, CAP40);", "return rescale(x, k);"),
    ("fraclen_off_by_one", "<= qmax_of(bits)) break;", "< qmax_of(bits)) break;"),
    ("fraclen_ignores_rounding", "if (rescale(m, -(ex + fl)) <= qmax_of(bits)) break;",
     "if (m * 2 <= (qmax_of(bits) * 2 + 1) * ((wide)1 << ((-(ex + fl)) > 0 && (-(ex+fl)) < 100 ? -(ex+fl) : 0)) && -(ex+fl) > 0) break;"),
    ("quantize_drops_sign", "rescale(neg ? -m : m, -(ex + fl))", "rescale(m, -(ex + fl))"),
    ("quantize_fl_sign", "rescale(neg ? -m : m, -(ex + fl))", "rescale(neg ? -m : m, -(ex - fl))"),
    ("vmax_window", "fl_default + DELTA_MAX) fl = fl_default + DELTA_MAX;", "fl_default + DELTA_MAX) fl = fl_default;"),
    ("comp_added_twice", "wide c  = comp ? load_q(comp, i, comp_bits) : 0;", "wide c  = comp ? 2 * load_q(comp, i, comp_bits) : 0;"),
    ("momentum_mu_grid", "rescale((wide)mu_q * m, (fl_m_in + 16) - G);", "rescale((wide)mu_q * m, fl_m_in - G);"),
    ("momentum_gradient_sign", "w += rescale_cap(-(wide)lr_q * g, (fl_g + 16) - G);", "w += rescale_cap((wide)lr_q * g, (fl_g + 16) - G);"),
    ("momentum_guard_bits", "wide mq = rescale(w, 16);", "wide mq = rescale(w, 15);"),
    ("momentum_step_grid", "wide s = rescale_cap(mn, fl_m_out - F);", "wide s = rescale_cap(mn, F - fl_m_out);"),
    ("momentum_old_velocity_used", "wide s = rescale_cap(mn, fl_m_out - F);", "wide s = rescale_cap(m, fl_m_out - F);"),
    ("momentum_decay_grid", "* th, (fl_in + 32) - G);", "* th, (fl_in + 16) - G);"),
    ("momentum_velocity_not_saturated", "wide mn = sat(mq, mom_bits);", "wide mn = mq;"),
    ("theta_unscaled", "wide v = th * ((wide)1 << d) + c + s;", "wide v = th + c + s;"),
    ("adam_betas_swapped", "wide wM = rescale((wide)b1_q * m,", "wide wM = rescale((wide)b2_q * m,"),
    ("adam_complement_forgotten", "rescale_cap((wide)(65536u - b1_q) * g,", "rescale_cap((wide)b1_q * g,"),
    ("adam_gradient_not_squared", "(wide)(65536u - b2_q) * g * g,", "(wide)(65536u - b2_q) * g,"),
    ("adam_square_grid", "(2 * fl_g + 16) - Gu);", "(fl_g + 16) - Gu);"),
    ("adam_root_grid_parity", "const int par = ((fl_u_out % 2) + 2) % 2;", "const int par = 0;"),
    ("adam_root_rounds_up", "if (t * t <= a) r = t;", "if (t * t < a) r = t + 1;"),
    ("adam_root_misses_squares", "if (t * t <= a) r = t;", "if (t * t < a) r = t;"),
    ("adam_eps_dropped", "wide den = rt + eps_R;", "wide den = rt;"),
    ("adam_step_sign", "wide num = -(wide)lr_q * mn;", "wide num = (wide)lr_q * mn;"),
    ("adam_old_moment_in_step", "wide num = -(wide)lr_q * mn;", "wide num = -(wide)lr_q * m;"),
    ("adam_division_truncates", "if (2 * r > den || (2 * r == den && (q & 1))) q += 1;", "if (0) q += 1;"),
    ("adam_division_ties_up", "if (2 * r > den || (2 * r == den && (q & 1))) q += 1;", "if (2 * r >= den) q += 1;"),
    ("adam_step_exponent", "const int e = F + R - 16 - (int)lr_exp - fl_m_out;", "const int e = F + R - 16 - (int)lr_exp + fl_m_out;"),
    ("adam_lr_exponent_ignored", "const int e = F + R - 16 - (int)lr_exp - fl_m_out;", "const int e = F + R - 16 - fl_m_out;"),
    ("adam_second_moment_goes_negative", "wide un = clampw(uq, 0, qmax_of(sec_bits));", "wide un = sat(uq, sec_bits);"),
    ("adam_moment_guard_bits", "wide uq = rescale(wU, 16);", "wide uq = rescale(wU, 15);"),
    ("momentum_mmax_truncates_the_guard_bits", "wide aw = mq < 0 ? -mq : mq;", "wide aw = (w < 0 ? -w : w) >> 16;"),
    ("empty_tensor_flagged", "if (n == 0) return LPK_REF_OK;", ""),
]

CHECKS = [
    lambda: bf.test_step_random_domain(0),
    bf.test_step_typical_shifts,
    bf.test_step_saturation_and_cap,
    lambda: bf.test_quantize_bruteforce(8),
    lambda: bf.test_fraclen_is_largest_non_saturating(8),
    lambda: bf.test_fraclen_from_vmax_bruteforce(16),
    lambda: pins.test_quarter_lsb_worked_example(+1),
    lambda: pins.test_conservation_invariant(8),
    pins.test_fraclen_hand_cases,
    pins.test_quantize_hand_cases,
    lambda: mom.test_momentum_step_bruteforce(0),
    mom.test_velocity_decay_and_fixed_point,
    mom.test_momentum_conserves_theta_plus_c,
    lambda: adam.test_adam_step_bruteforce(0),
    adam.test_constant_gradient_moves_theta_by_lr_per_step,
    adam.test_against_float64_adam,
    readings.test_an_empty_tensor_is_a_no_op_whatever_the_fraclens_hold,
    readings.test_velocity_exponent_comes_from_the_rounded_velocity_at_a_power_of_two_boundary,
]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(name, old, new, tmp_path, monkeypatch):
    text = open(SRC).read()
    assert text.count(old) >= 1, "mutation anchor must match the oracle source: %r" % old
    c = tmp_path / "mut.c"
    so = tmp_path / ("mut_%s.so" % name)
    c.write_text(text.replace(old, new, 1))        # the first match (the plain update comes first in the file)
    subprocess.check_call(["gcc", "-O1", "-w", "-shared", "-fPIC", "-o", str(so), str(c), "-lm"])
    monkeypatch.setattr(ref, "_lib", ref.load(str(so)))
    caught = False
    order = CHECKS[::-1] if name.startswith(("adam", "momentum")) else CHECKS      # likeliest catchers first: same verdict, sooner
    for chk in order:
        try:
            chk()
        except AssertionError:
            caught = True
            break
    assert caught, "mutation %s survived every pin" % name

"""The pins must be able to fail: each planted mistake in a *copy* of the oracle's C source (never in
the HIP path) has to be rejected by the CPU pin tests.  Runs on the CPU only."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "lutkan_oracle.c")

MUTATIONS = {
    "lerp_weights_swapped": ("float p0 = omw * v0;\n    float p1 = w * v1;", "float p0 = w * v0;\n    float p1 = omw * v1;"),
    "dequant_drops_y_min": ("float v0 = y_min + a0;", "float v0 = a0;"),
    "searchsorted_left": ("if (T[kappa] <= xc) ++cnt;", "if (T[kappa] < xc) ++cnt;"),
    "lookup_uses_L_not_L_minus_1": ("float z = u * (float)(L - 1);", "float z = u * (float)(L);"),
    "sampling_closed_grid": ("/ (double)L;", "/ (double)(L - 1);"),
    "symmetric_uses_128": ("float a = amax / 127.0f;", "float a = amax / 128.0f;"),
    "recursion_wrong_right_denominator": ("double dr = tau[r + q + 1] - tau[r + 1];", "double dr = tau[r + q + 1] - tau[r];"),
    "recursion_wrong_left_numerator": ("(x - tau[r]) / dl * N[r]", "(x - tau[r + 1]) / dl * N[r]"),
    "closed_mode_excludes_tK": ("(uint8_t)(x >= t0 && x <= tK)", "(uint8_t)(x >= t0 && x < tK)"),
    "half_open_includes_tK": (": (uint8_t)(x >= t0 && x < tK);", ": (uint8_t)(x >= t0 && x <= tK);"),
    "zero_spline_ignored": ("(oob == LKO_ZERO_SPLINE && !ix.in) ? 0.0f : v;", "v;"),
    "edge_index_transposed": ("size_t e = (size_t)i * m + j;\n                size_t seg", "size_t e = (size_t)j * d + i;\n                size_t seg"),
    "round_half_away": ("float r = rintf(t / a);", "float r = roundf(t / a);"),
    "no_nextafter": ("nextafterf(tK, -INFINITY)", "tK"),
    "l1_not_clamped_to_l0_plus_1": ("o->l1 = (l0 + 1 < L - 1) ? l0 + 1 : L - 1;", "o->l1 = l0;"),
    "asym_min_is_zero": ("*y_min = lo;", "*y_min = 0.0f;"),
    "degree0_closed_indicator": ("(tau[r] <= x && x < tau[r + 1])", "(tau[r] <= x && x <= tau[r + 1])"),
    "base_branch_at_clipped_x": ("const float silu_x = edge_out ? lko_silu(x[(size_t)b * d + i]) : 0.0f;", "const float silu_x = edge_out ? lko_silu(ix.xc) : 0.0f;"),
    "silu_wrong_sign": ("return (float)(xd / (1.0 + exp(-xd)));", "return (float)(xd / (1.0 + exp(xd)));"),
    "edge_output_scale_dropped": ("float phi = s_out * sum;", "float phi = sum;"),
    "spline_scale_on_base": ("float tb = s_base * b;\n    float ts = s_spline * spline_term;", "float tb = s_spline * b;\n    float ts = s_base * spline_term;"),
    "bspline_layer_masks_base_too": ("                if (masked) { s = 0.0; sa = 0.0; }\n                if (edge_out) {", "                if (edge_out) {"),
    "fp16_params_truncated": ("double r = nearbyint(a / ulp) * ulp;", "double r = floor(a / ulp) * ulp;"),
    "fp16_params_no_subnormals": ("if (lead < -14) lead = -14;", "if (lead < -24) lead = -24;"),
    "fp16_params_overflow_late": ("if (a >= 65520.0) return", "if (a > 65535.0) return"),
    "extended_lut_drops_last_interval": ("int K = extended ? n - 1 : G;                        /* LUT segments", "int K = extended ? n - 2 : G;                        /* LUT segments"),
    "extended_layer_keeps_inner_domain": ("T_all[h][k] = extended ? tau_f[(size_t)h * n + k] :", "T_all[h][k] = extended ? tau_f[(size_t)h * n + (k < p ? p : (k > p + G ? p + G : k))] :"),
    "layer_sum_skips_first_input": ("for (int i = 0; i < d; ++i) {\n            lko_index ix;\n            lko_locate(knots", "for (int i = (d > 1); i < d; ++i) {\n            lko_index ix;\n            lko_locate(knots"),
    "per_input_forward_uses_first_vector": ("lko_locate(knots + (per_input ? (size_t)i * (K + 1) : 0),", "lko_locate(knots + (per_input ? (size_t)0 * (K + 1) : 0),"),
    "per_input_compile_uses_first_vector": ("const double *Bh = Bs + (per_input ? (size_t)(e / m) : 0) * K * L * n;", "const double *Bh = Bs;"),
    "per_input_compile_indexes_by_output": ("const double *Bh = Bs + (per_input ? (size_t)(e / m) : 0) * K * L * n;", "const double *Bh = Bs + (per_input ? (size_t)((e % m) % d) : 0) * K * L * n;"),
    "per_input_bspline_uses_first_vector": ("const double *tau = tau_all[per_input ? i : 0];", "const double *tau = tau_all[0];"),
    "per_input_bspline_domain_of_first_vector": ("lko_locate(T_all[per_input ? i : 0], K, 2,", "lko_locate(T_all[0], K, 2,"),
}


def test_every_mutation_text_is_present_once():
    src = open(SRC).read()
    for name, (old, _) in MUTATIONS.items():
        assert src.count(old) == 1, name        # (two mutations may share one site)


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_pins_reject_planted_mistake(name, tmp_path):
    old, new = MUTATIONS[name]
    src = open(SRC).read().replace(old, new)
    msrc = tmp_path / "mutant.c"
    msrc.write_text(src)
    env = dict(os.environ, LUTKAN_ORACLE_SRC=str(msrc), LUTKAN_ORACLE_LIB=str(tmp_path / "libmutant.so"))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_bspline.py"),
                        os.path.join(ROOT, "tests", "test_oracle_lut.py")],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 1, f"mutation {name} survived the pins:\n{r.stdout[-2000:]}"

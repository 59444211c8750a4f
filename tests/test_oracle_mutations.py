"""Do the oracle's pins bite?  Each case plants one plausible mistake in a COPY of the oracle's C source (on the
CPU, never in the product), builds it, swaps it in for the real oracle and re-runs pins from the other test
modules: at least one of them must fail.  The unmodified copy must pass the same pins."""
import ctypes as C
import os
import subprocess
import tempfile

import pytest

from oracle import oracle as O
from tests import test_oracle_decoder as D
from tests import test_oracle_schedule as Sch

SRC = open(os.path.join(os.path.dirname(O.__file__), "skd_oracle.c")).read()

MUTATIONS = {
    # name: (original text, replacement)
    "schedule_floor_instead_of_half_up": ("return (int)((twice_r_times_T + T) / (2 * T));", "return (int)(twice_r_times_T / (2 * T));"),
    "schedule_prompt_at_n_max": ("if (i < P) return L;", "if (i < P) return n_max;"),
    "window_at_the_bottom": ("for (int l = L - top; l < L; ++l) out[c++] = l;", "for (int l = warmup; l < warmup + top; ++l) out[c++] = l;"),
    "ln_unbiased_variance": ("var /= (real)d;", "var /= (real)(d - 1);"),
    "ln_missing_bias": ("* (real)g[k] + (real)b[k];", "* (real)g[k];"),
    "linear_missing_bias": ("out[(size_t)r * N + o] = acc + (bias ? (real)bias[o] : (real)0);", "out[(size_t)r * N + o] = acc;"),
    "attention_scale_1_over_dh": ("real inv = (real)1 / (real)sqrt((double)dh);", "real inv = (real)1 / (real)dh;"),
    "attention_no_max_subtraction_sign": ("scratch[j] = (real)exp((double)(scratch[j] - mx));", "scratch[j] = (real)exp((double)(mx - scratch[j]));"),
    "values_taken_from_keys": ("Vd[k] = qkv[(size_t)b * 3 * d + 2 * d + k];", "Vd[k] = qkv[(size_t)b * 3 * d + d + k];"),
    "ffn_residual_dropped": ("linear(w->w2[l], w->b2[l], u, B, f, d, t1);\n    for (size_t k = 0; k < (size_t)B * d; ++k) x[k] += t1[k];",
                             "linear(w->w2[l], w->b2[l], u, B, f, d, t1);\n    for (size_t k = 0; k < (size_t)B * d; ++k) x[k] = t1[k];"),
    "relu_dropped": ("for (size_t k = 0; k < (size_t)B * f; ++k) u[k] = u[k] > 0 ? u[k] : 0;", "/* no relu */"),
    "position_ignores_padding": ("if (is_real) st->n_real[b] += 1;", "st->n_real[b] += 1;"),
    "padding_keys_not_masked": ("      if (!valid[j]) continue;\n", ""),
    "heads_share_first_head_query": ("s += q[h * dh + e] * Kc[(size_t)j * d + h * dh + e];", "s += q[e] * Kc[(size_t)j * d + h * dh + e];"),
    "final_layernorm_skipped": ("for (int b = 0; b < B; ++b) layernorm(x + (size_t)b * d, w->lnf_g, w->lnf_b, d, a1 + (size_t)b * d);\n    linear(w->lm_head",
                                "for (size_t k = 0; k < (size_t)B * d; ++k) a1[k] = x[k];\n    linear(w->lm_head"),
    "argmax_takes_last_on_ties": ("if (z[(size_t)b * V + v] > z[(size_t)b * V + best]) best = v;", "if (z[(size_t)b * V + v] >= z[(size_t)b * V + best]) best = v;"),
    "sampling_excludes_ties": ("if (p[i] >= tau) mass += p[i];", "if (p[i] > tau || (p[i] == tau && i == 0)) mass += p[i];"),
}

PINS = [Sch.test_fig3_worked_example, Sch.test_table2_target_average, Sch.test_properties_random,
        Sch.test_active_set_is_top_window_and_warmup, Sch.test_contract_config_sums,
        D.test_full_depth_equals_textbook_decoder, D.test_left_padding_matches_unpadded_row,
        D.test_skipped_layers_are_dead_and_top_layers_matter, D.test_sampling_head_pins, D.test_ops_against_library,
        lambda: D.test_skip_equals_prefix_form_and_bruteforce(2, 3, 1, 4, 12),
        D.test_argmax_lowest_index_on_ties]


def _build(src, tag, tmp):
    path = os.path.join(tmp, f"ora_{tag}.c")
    open(path, "w").write(src)
    out = os.path.join(tmp, f"libora_{tag}.so")
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-DORA_REAL=double", path, "-o", out, "-lm"],
                   check=True)
    return out


def _run_pins():
    failed = []
    for pin in PINS:
        try:
            pin()
        except (AssertionError, O.OracleError) as e:
            failed.append(getattr(pin, "__name__", "pin"))
    return failed


@pytest.fixture(scope="module")
def tmpdir_mod():
    with tempfile.TemporaryDirectory() as t:
        yield t


def _swap_in(path):
    real = O._lib("f64")
    O._LIBS.pop("f64")
    old_build = O.build
    O.build = lambda r="f64", force=False: path if r == "f64" else old_build(r, force)
    O._lib("f64")
    return real, old_build


def _swap_out(real, old_build):
    O.build = old_build
    O._LIBS["f64"] = real


def test_unmodified_copy_passes(tmpdir_mod):
    saved = _swap_in(_build(SRC, "clean", tmpdir_mod))
    try:
        assert _run_pins() == []
    finally:
        _swap_out(*saved)


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name, tmpdir_mod):
    old, new = MUTATIONS[name]
    assert SRC.count(old) >= 1, f"mutation site for {name} not found"
    saved = _swap_in(_build(SRC.replace(old, new), name, tmpdir_mod))
    try:
        failed = _run_pins()
    finally:
        _swap_out(*saved)
    assert failed, f"no pin noticed: {name}"

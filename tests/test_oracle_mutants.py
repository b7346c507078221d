"""Are the pins sharp?  Each plausible mistake (a dropped factor, a wrong sign or index, a transposed
operand, a swapped constant) is planted in a copy of the oracle's C source, compiled, and run against
the pin tests of test_oracle_pins.py; every mutant must fail at least one pin, and the unmodified
source must pass them all.  CPU only: nothing here touches the GPU library."""
import os
import subprocess

import pytest

import oracle
import test_oracle_pins as P

SRC = os.path.join(os.path.dirname(oracle.__file__), "normtest_oracle.c")

# (name, text to find, replacement[, which occurrence]): without the fourth entry `find` must occur exactly once
MUTANTS = [
    ("mean_not_divided", "gbar = s / (double)J;\n    for (int64_t j = 0; j < J; ++j) {\n      double r", "gbar = s;\n    for (int64_t j = 0; j < J; ++j) {\n      double r", 0),
    ("coord_mean_not_divided", "gbar = s / (double)J;\n    for (int64_t j = 0; j < J; ++j) {\n      double r", "gbar = s;\n    for (int64_t j = 0; j < J; ++j) {\n      double r", 1),
    ("B_not_squared", "csum_add(acc + 2, s * s);", "csum_add(acc + 2, s);"),
    ("residual_not_squared", "c += r * r;", "c += r;", 0),
    ("coord_residual_not_squared", "c += r * r;", "c += r;", 1),
    ("A_not_squared", "a += g * g;", "a += g;"),
    ("transposed_index", "double g = widen(grads, dtype, j * ld + i);", "double g = widen(grads, dtype, i * J + j);"),
    ("residual_other_row", "double r = widen(grads, dtype, j * ld + i) - gbar;", "double r = widen(grads, dtype, i) - gbar;", 0),
    ("coord_residual_other_row", "double r = widen(grads, dtype, j * ld + i) - gbar;", "double r = widen(grads, dtype, i) - gbar;", 1),
    ("bf16_shift", "u = (uint32_t)h << 16;", "u = (uint32_t)h << 15;"),
    ("gbar_sq_over_J", "out->gbar_sq = B / (Jd * Jd);", "out->gbar_sq = B / Jd;"),
    ("ddof_ignored", "out->var_l1 = C / (double)(J - ddof);", "out->var_l1 = C / (double)J;"),
    ("ddof_doubled", "out->var_l1 = C / (double)(J - ddof);", "out->var_l1 = C / (double)(J - 2 * ddof + 1);"),
    ("eta_not_squared", "T = out->var_l1 / (eta * eta * out->gbar_sq);", "T = out->var_l1 / (eta * out->gbar_sq);"),
    ("T_inverted", "T = out->var_l1 / (eta * eta * out->gbar_sq);", "T = (eta * eta * out->gbar_sq) / out->var_l1;"),
    ("equality_grows", "if (T > (double)b_k) {", "if (T >= (double)b_k) {"),
    ("floor_not_ceil", "int64_t t = (int64_t)ceil(T);", "int64_t t = (int64_t)floor(T);"),
    ("round_down", "int64_t q = t / round_to + (t % round_to != 0);", "int64_t q = t / round_to;"),
    ("round_up_always", "int64_t q = t / round_to + (t % round_to != 0);", "int64_t q = t / round_to + 1;"),
    ("no_cap", "if (b_max > 0 && nb > b_max) {", "if (0) {"),
    ("cap_may_shrink", "if (nb < b_k) nb = b_k;", ""),
    ("zero_norm_passes", "out->T = INFINITY;\n      out->pass = 0;", "out->T = INFINITY;\n      out->pass = 1;"),
    ("m_weights_swapped", "mn = beta1 * (double)m[i] + (1.0 - beta1) * g;", "mn = (1.0 - beta1) * (double)m[i] + beta1 * g;"),
    ("v_not_squared", "vn = beta2 * (double)v[i] + (1.0 - beta2) * g * g;", "vn = beta2 * (double)v[i] + (1.0 - beta2) * g;"),
    ("scale_ignored", "g = grad_scale * gbar;", "g = gbar;"),
    ("scale_only_first_moment", "vn = beta2 * (double)v[i] + (1.0 - beta2) * g * g;", "vn = beta2 * (double)v[i] + (1.0 - beta2) * gbar * gbar;"),
    ("coord_rhs_without_batch", "rhs = eta * eta * (double)b_k * gbar * gbar;", "rhs = eta * eta * gbar * gbar;"),
    ("coord_rhs_mean_not_squared", "rhs = eta * eta * (double)b_k * gbar * gbar;", "rhs = eta * eta * (double)b_k * gbar;"),
    ("coord_ddof_ignored", "var = c / (double)(J - ddof);", "var = c / (double)J;"),
    ("coord_equality_fails", "if (var > rhs * (1.0 + band))", "if (var >= rhs * (1.0 + band))"),
    ("coord_inequality_flipped", "if (var > rhs * (1.0 + band))", "if (var < rhs * (1.0 + band))"),
    ("ratio_without_batch", "rho = variance / (eta * eta * (double)b_k * mean * mean);", "rho = variance / (eta * eta * mean * mean);"),
    ("ratio_eta_not_squared", "rho = variance / (eta * eta * (double)b_k * mean * mean);", "rho = variance / (eta * (double)b_k * mean * mean);"),
    ("ratio_mean_not_squared", "rho = variance / (eta * eta * (double)b_k * mean * mean);", "rho = variance / (eta * eta * (double)b_k * mean);"),
    ("ratio_inverted", "rho = variance / (eta * eta * (double)b_k * mean * mean);", "rho = (eta * eta * (double)b_k * mean * mean) / variance;"),
    ("ratio_ddof_ignored", "variance = spread / (double)(J - ddof);", "variance = spread / (double)J;"),
    ("ratio_minimum", "if (rho > *out) *out = rho;", "if (rho < *out) *out = rho;"),
    ("ratio_last_not_largest", "if (rho > *out) *out = rho;", "*out = rho;"),
    ("ratio_zero_mean_ignored", "else if (mean == 0.0)\n      rho = INFINITY;", "else if (mean == 0.0)\n      rho = 0.0;"),
    ("ratio_no_spread_is_nan", "if (variance == 0.0)\n      rho = 0.0;\n    else if", "if (0)\n      rho = 0.0;\n    else if"),
    ("ratio_mean_not_divided", "mean = total / (double)J;", "mean = total;"),
    ("ratio_deviation_not_squared", "spread += dev * dev;", "spread += dev;"),
    ("resplit_ignores_cap", "if (m < M_base) m = M_base;", "m = M_base;"),
    ("resplit_floor_micro", "mb = b / (J * m) + (b % (J * m) != 0);", "mb = b / (J * m);"),
    ("resplit_steps_from_total", "m = per_worker / micro_max + (per_worker % micro_max != 0);", "m = b / micro_max + (b % micro_max != 0);"),
    ("due_counts_from_zero", "return (step - 1) % interval == 0 ? 1 : 0;", "return step % interval == 0 ? 1 : 0;"),
    ("due_ignores_interval", "return (step - 1) % interval == 0 ? 1 : 0;", "return 1;"),
    ("due_ignores_maximum", "if (b_max > 0 && b_k >= b_max) return 0;", ""),
    ("due_strictly_above_maximum", "if (b_max > 0 && b_k >= b_max) return 0;", "if (b_max > 0 && b_k > b_max) return 0;"),
    ("due_zero_maximum_stops", "if (b_max > 0 && b_k >= b_max) return 0;", "if (b_k >= b_max) return 0;"),
    ("clip_never", "return c < 1.0 ? c : 1.0;", "return 1.0;"),
    ("clip_always", "return c < 1.0 ? c : 1.0;", "return c;"),
    ("clip_uses_squared_norm", "c = max_norm / (sqrt(gbar_sq) + 1e-6);", "c = max_norm / (gbar_sq + 1e-6);"),
    ("bias1_uses_beta2", "bc1 = 1.0 - pow(beta1, (double)step);", "bc1 = 1.0 - pow(beta2, (double)step);"),
    ("bias2_missing", "vhat = vn / bc2;", "vhat = vn;"),
    ("bias1_missing", "mhat = mn / bc1;", "mhat = mn;"),
    ("eps_inside_root", "lr * mhat / (sqrt(vhat) + eps);", "lr * mhat / sqrt(vhat + eps);"),
    ("no_weight_decay", "w_out[i] = (1.0 - lr * wd) * (double)w[i]", "w_out[i] = (double)w[i]"),
    ("decay_not_scaled_by_lr", "w_out[i] = (1.0 - lr * wd) * (double)w[i]", "w_out[i] = (1.0 - wd) * (double)w[i]"),
    ("update_sign", "(double)w[i] - lr * mhat", "(double)w[i] + lr * mhat"),
    ("adamw_mean_not_divided", "gbar = s / (double)J;\n    g =", "gbar = s;\n    g ="),
    ("compensation_dropped", "s[1] += (s[0] - t) + x;", "s[1] += 0.0;"),
]


def battery():
    """The pins, cheapest first.  Each entry raises AssertionError when the oracle under test is wrong."""
    stat_cases = [c for c in P.GOLDEN_CASES if "expect_A" in c]
    adam_cases = [c for c in P.GOLDEN_CASES if "expect_w" in c]
    checks = []
    for c in stat_cases:
        for b in (False, True):
            checks.append(lambda c=c, b=b: P.test_golden_statistic(c, b))
    for c in adam_cases:
        checks.append(lambda c=c: P.test_golden_adamw(c))
    for c in [c for c in P.GOLDEN_CASES if any(k.startswith("coord_") for k in c)]:
        checks.append(lambda c=c: P.test_golden_coordinatewise(c, False))
    for J, d, b in ((3, 3, False), (4, 16, True), (5, 1, False), (8, 16, False)):
        checks.append(lambda J=J, d=d, b=b: P.test_brute_force_exact_rational(J, d, b))
    checks += [
        P.test_equality_passes_and_strict_excess_grows,
        lambda: P.test_rounding_chain_against_alg1_lines(4, 16),
        lambda: P.test_rounding_chain_against_alg1_lines(3, 5),
        P.test_degenerate_inputs,
        P.test_ddof_relation,
        P.test_row_stride_is_honoured,
        P.test_matches_library_adamw_over_steps,
        P.test_adamw_first_step_is_a_sign_step,
        lambda: P.test_matches_numpy_column_variance(7, 1),
        lambda: P.test_identity_C_equals_A_minus_B_over_J(7, P.torch.bfloat16),
        lambda: P.test_zero_variance_when_rows_identical(4),
        P.test_scale_row_permutation_and_shard_additivity,
        P.test_long_sum_needs_compensation,
        P.test_clipped_step_matches_library_clipping,
        lambda: P.test_coordinatewise_brute_force_and_invariants(3),
        P.test_resplit_reproduces_the_papers_table_values_and_invariants,
        P.test_test_schedule_interval_and_maximum,
    ]
    return checks


def first_failure(checks):
    for k, chk in enumerate(checks):
        try:
            chk()
        except AssertionError:
            return k
    return None


def compile_variant(src_text: str, out_path: str, extra=()) -> str:
    c_path = out_path[:-3] + ".c"
    with open(c_path, "w") as f:
        f.write(src_text)
    subprocess.run(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fno-fast-math", "-ffp-contract=off", *extra,
                    "-o", out_path, c_path, "-lm"], check=True)
    return out_path


@pytest.fixture
def swap_oracle(monkeypatch):
    def use(path):
        monkeypatch.setattr(oracle, "_lib", oracle._bind(path))
    return use


def test_unmodified_source_passes_every_pin(tmp_path, swap_oracle):
    swap_oracle(compile_variant(open(SRC).read(), str(tmp_path / "clean.so")))
    assert first_failure(battery()) is None


def test_oracle_is_clean_under_the_undefined_behaviour_sanitizer(tmp_path, swap_oracle, capfd):
    """The whole pin battery on a -fsanitize=undefined build of the oracle: no report may be printed."""
    swap_oracle(compile_variant(open(SRC).read(), str(tmp_path / "ubsan.so"), extra=("-g", "-fsanitize=undefined")))
    assert first_failure(battery()) is None
    err = capfd.readouterr().err
    assert "runtime error" not in err, err


def plant(text: str, find: str, repl: str, which=None) -> str:
    if which is None:
        assert text.count(find) == 1, "mutation target must occur exactly once: %r" % find
        return text.replace(find, repl)
    pos = -1
    for _ in range(which + 1):
        pos = text.index(find, pos + 1)
    return text[:pos] + repl + text[pos + len(find):]


@pytest.mark.parametrize("mutant", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_each_planted_mistake_is_caught(mutant, tmp_path, swap_oracle):
    name, find, repl = mutant[:3]
    text = plant(open(SRC).read(), find, repl, mutant[3] if len(mutant) > 3 else None)
    swap_oracle(compile_variant(text, str(tmp_path / (name + ".so"))))
    assert first_failure(battery()) is not None, "no pin noticed the planted mistake %r" % name

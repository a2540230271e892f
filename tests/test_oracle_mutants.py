"""Do the pins pin?  Each case plants one plausible mistake in a copy of the oracle's C source (a
dropped term, a wrong sign or index, a swapped operand), builds it, and runs the oracle's pin tests
against the broken build in a child process: they must fail.  Nothing here touches the GPU or the
GPU library; the mistakes live in a temporary copy only."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "ears_oracle.c")
PINS = ["tests/test_oracle_rng.py", "tests/test_oracle_rules.py", "tests/test_oracle_greedy.py",
        "tests/test_oracle_lm_head.py"]

# (name, text in the oracle, planted mistake, pin files that must notice)
MUTANTS = [
    ("philox_rounds", "round < 10;", "round < 9;", PINS[:1]),
    ("philox_multipliers_swapped", "(uint64_t)0xD2511F53u * (uint64_t)c0", "(uint64_t)0xCD9E8D57u * (uint64_t)c0", PINS[:1]),
    ("philox_key_not_bumped", "    k1 += 0xBB67AE85u;\n", "", PINS[:1]),
    ("philox_words_misplaced", "uint32_t n1 = lo1;", "uint32_t n1 = lo0;", PINS[:1]),
    ("uniform_23_bits", "(double)(w >> 8) * 0x1p-24", "(double)(w >> 9) * 0x1p-24", PINS[:1]),
    ("gumbel_coarse_byte_order", "(8u * (v & 3u))", "(8u * (3u - (v & 3u)))", PINS[:1]),
    ("gumbel_no_half_step", "((double)f + 0.5)", "((double)f)", PINS[:1]),
    ("gumbel_sign", "return -log(-log(u));", "return log(-log(u));", PINS[:2]),
    ("temperature_dropped", "- m) / T);", "- m));", PINS[1:2]),
    ("temperature_inverted", "- m) / T);", "- m) * T);", PINS[1:2]),
    ("uncertainty_is_max_probability", "double unc = 1.0 - maxpt;", "double unc = maxpt;", PINS[1:2]),
    ("ratio_inverted", "double R = Ptx / Pd_safe;", "double R = Pd_safe / fmax(Ptx, 1e-300);", PINS[1:2]),
    ("guard_on_target", "double Pd_safe = (Pdx > 1e-10) ? Pdx : 1e-10;",
     "double Pd_safe = Pdx; if (Ptx < 1e-10) Ptx = 1e-10;", PINS[1:2]),
    ("tolerance_added_to_threshold", "double thr = U - tol;", "double thr = U + tol;", PINS[1:2]),
    ("tolerance_ignores_uncertainty", "double tol = beta * unc;", "double tol = beta;", PINS[1:2]),
    ("strict_comparison", "} else if (R >= thr) {", "} else if (R > thr) {", PINS[1:2]),
    ("accept_length_off_by_one", "      n = i; /* x_i", "      n = i + 1; /* x_i", PINS[1:2]),
    ("later_rejection_wins", "if (decision == 0 && !first_reject_seen) {", "if (decision == 0) {", PINS[1:2]),
    ("residual_sign", "      double q = pt[v] - pd[v];\n", "      double q = pd[v] - pt[v];\n", PINS[1:2]),
    ("residual_support_without_floor", "if (q <= EARS_ORACLE_RESIDUAL_FLOOR * (pt[v] + pd[v])) q = 0.0;", "", PINS[1:2]),
    ("replacement_from_target", "      double q = pt[v] - pd[v];\n", "      double q = pt[v];\n", PINS[1:2]),
    ("bonus_row", "const void* row = row_ptr(target_rows, dtype, K, V);",
     "const void* row = row_ptr(target_rows, dtype, K - 1, V);", PINS[1:2]),
    ("bonus_ignores_temperature", "top2_push(&top, l / T + ears_oracle_gumbel", "top2_push(&top, l + ears_oracle_gumbel", PINS[1:2]),
    ("argmax_ties_to_highest_index", "if (t->arg < 0 || s > t->best) {", "if (t->arg < 0 || s >= t->best) {", PINS[1:2]),
    ("runner_up_not_updated_by_new_winner", "    t->second = (t->arg < 0) ? -INFINITY : t->best;\n    t->arg2 = t->arg;\n", "", PINS[1:2]),
    ("runner_up_index_stale", "    t->second = s;\n    t->arg2 = v;\n", "    t->second = s;\n", PINS[1:2]),
    ("runner_up_ties_to_highest_index", "} else if (t->arg2 < 0 || s > t->second) {", "} else if (t->arg2 < 0 || s >= t->second) {", PINS[1:2]),
    ("gap_of_winner_with_itself", "samp[2] = t->best - t->second;", "samp[2] = t->best - t->best;", PINS[1:2]),
    ("entropy_in_bits", "H -= p[v] * log(p[v]);", "H -= p[v] * log2(p[v]);", PINS[1:2]),
    ("variance_is_sum_of_squares", "G += p[v] * (1.0 - p[v]);", "G += p[v] * p[v];", PINS[1:2]),
    ("variance_measure_not_selected", "    if (unc_mode == EARS_ORACLE_UNC_VARIANCE) unc = ears_oracle_variance(pt, V);\n", "", PINS[1:2]),
    ("ragged_target_rows", "row_ptr(target, dtype, r0 + b, V), row_ptr(draft, dtype, r0, V), tokens + r0",
     "row_ptr(target, dtype, r0, V), row_ptr(draft, dtype, r0, V), tokens + r0", PINS[1:2]),
    ("greedy_ties_to_highest_index", "    if (x > bv) {", "    if (x >= bv) {", PINS[2:3]),
    ("greedy_keeps_matching_after_mismatch", "if (i < Kb && n == Kb && tokens[r0 + i] != a) n = i;",
     "if (i < Kb && tokens[r0 + i] != a) n = i;", PINS[2:3]),
    ("greedy_token_from_previous_row", "i < n ? tokens[r0 + i] : (i == n ? a : -1)",
     "i < n ? tokens[r0 + i] : (i == n ? tokens[r0 + (i < Kb ? i : Kb - 1)] : -1)", PINS[2:3]),
    ("projection_wrong_hidden_row", "bf16_value(hidden[(size_t)n * D + k])", "bf16_value(hidden[(size_t)k])", PINS[3:4]),
    ("projection_wrong_weight_row", "bf16_value(weight[(size_t)v * D + k])", "bf16_value(weight[(size_t)n * D + k])", PINS[3:4]),
    ("bf16_truncates", "double q = nearbyint(ldexp(m, 8));", "double q = floor(ldexp(m, 8));", PINS[3:4]),
    ("bf16_ties_away", "double q = nearbyint(ldexp(m, 8));", "double q = round(ldexp(m, 8));", PINS[3:4]),
]


@pytest.mark.parametrize("name,old,new,pins", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, old, new, pins):
    src = open(SRC).read()
    assert src.count(old) == 1, "the oracle no longer contains this text exactly once: %r" % old
    mutant_c = tmp_path / "mutant.c"
    mutant_c.write_text(src.replace(old, new))
    (tmp_path / "ears_oracle.h").write_text(open(os.path.join(ROOT, "oracle", "ears_oracle.h")).read())
    lib = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                           "-w", "-o", str(lib), str(mutant_c), "-lm"])
    env = dict(os.environ, EARS_ORACLE_LIB=str(lib))
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + pins,
                         cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=300)
    assert run.returncode != 0, "no pin noticed the planted mistake '%s'" % name
    assert b"failed" in run.stdout or b"error" in run.stdout.lower()

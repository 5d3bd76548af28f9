"""The pins must catch a plausible mistake anywhere in the oracle.  Each case plants ONE mistake
(a wrong sign, a dropped term, '<' for '<=', a wrong constant ...) in a copy of the oracle's
sources, builds it, and runs the pin tests against that build in a subprocess: they must fail.
CPU only; the mistakes live in a temporary directory, never in the repository."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE = os.path.join(ROOT, "oracle")
PIN_TESTS = ["tests/test_oracle_pins.py", "tests/test_oracle_alns_pins.py", "tests/test_oracle_swap_pins.py",
             "tests/test_oracle_l2_pins.py"]

# (name, file, correct text, planted mistake)
MUTANTS = [
    ("residual_sign_of_b", "dmmv_oracle_impl.inc", "r[i] = FMA(acc, sc, -b[i]);", "r[i] = FMA(acc, sc, b[i]);"),
    ("step_sign", "dmmv_oracle_impl.inc", "REAL diff = D[k] - D[kcur];", "REAL diff = D[kcur] - D[k];"),
    ("radius_off_by_one", "dmmv_oracle_impl.inc", "if (d > radius) return 0;", "if (d >= radius) return 0;"),
    ("argmin_takes_last_of_ties", "dmmv_oracle_impl.inc", "if (c < 0 || scores[q] < s) { s = scores[q]; c = q; }",
     "if (c < 0 || scores[q] <= s) { s = scores[q]; c = q; }"),
    ("apply_without_fma_operand", "dmmv_oracle_impl.inc",
     "for (int64_t i = 0; i < m; ++i) r[i] = FMA(delta, Acol[i], r[i]);",
     "for (int64_t i = 0; i < m; ++i) r[i] = FMA(delta, Acol[i], -r[i]);"),
    ("descent_accepts_equal_scores", "dmmv_oracle_impl.inc",
     "        if (c < 0 || !(s < t)) break;\n        int64_t j = c / nd; int32_t k = (int32_t)(c % nd);\n        REAL delta = SFX(delta_of)(D, kidx[j], k, sc);",
     "        if (c < 0 || !(s <= t)) break;\n        int64_t j = c / nd; int32_t k = (int32_t)(c % nd);\n        REAL delta = SFX(delta_of)(D, kidx[j], k, sc);"),
    ("mix_constant", "alns_common.inc", "0xbf58476d1ce4e5b9ULL", "0xbf58476d1ce4e5b8ULL"),
    ("exp_coefficient", "alns_common.inc", "p = fma(p, w, 1.0 / 720.0);", "p = fma(p, w, 1.0 / 721.0);"),
    ("sample_boundary", "alns_common.inc", "if (prefix[mid] > v) hi = mid; else lo = mid + 1;",
     "if (prefix[mid] >= v) hi = mid; else lo = mid + 1;"),
    ("impact_slack_sign", "alns_oracle_impl.inc", "const double R = (t - sk) / a;", "const double R = (t + sk) / a;"),
    ("greedy_tie_goes_up", "alns_oracle_impl.inc", "knew = ehi < elo ? kc + 1 : kc - 1;", "knew = ehi <= elo ? kc + 1 : kc - 1;"),
    ("acceptance_strict", "alns_oracle_impl.inc", "const int accepted = t <= t_cur &&", "const int accepted = t < t_cur &&"),
    ("sumsq_drops_blocks", "alns_oracle_impl.inc", "        total += acc;", "        total = acc;"),
    ("swap_difference_reversed", "swap_oracle_impl.inc",
     "        const REAL d = aj[k] - ai[k];\n        const REAL v = FABS(FMA(Delta, d, r[k]));",
     "        const REAL d = ai[k] - aj[k];\n        const REAL v = FABS(FMA(Delta, d, r[k]));"),
    ("swap_allows_equal_values", "swap_oracle_impl.inc",
     "    if (!(kidx[i] > kidx[j])) return (REAL)INFINITY;", "    if (!(kidx[i] >= kidx[j])) return (REAL)INFINITY;"),
    ("swap_not_strict", "swap_oracle_impl.inc", "if (tp < t_best) { t_best = tp; best = i * n + j; }",
     "if (tp <= t_best) { t_best = tp; best = i * n + j; }"),
    ("swap_moves_one_value_only", "swap_oracle_impl.inc", "    kidx[j] = ki;\n", "    kidx[j] = kidx[j];\n"),
    ("mask_ignored", "dmmv_oracle_impl.inc", "if (var_mask && !var_mask[j]) return 0;", "if (var_mask && !var_mask[j]) return 1;"),
    ("dense_transposed_operand", "dmmv_oracle_impl.inc", "REAL v = FABS(FMA(delta, A[i + lda * j], r[i]));",
     "REAL v = FABS(FMA(delta, A[j + lda * i], r[i]));"),
    ("sparse_rest_over_all_rows", "dmmv_oracle_impl.inc",
     "        for (int64_t i = 0; i < m; ++i)\n            if (!touched[i]) { REAL a = FABS(r[i]); if (a > rest) rest = a; }\n        for (int32_t k = 0; k < nd; ++k) {",
     "        for (int64_t i = 0; i < m; ++i)\n            { REAL a = FABS(r[i]); if (a > rest) rest = a; }\n        for (int32_t k = 0; k < nd; ++k) {"),
    ("sorted_rest_takes_a_touched_row", "dmmv_oracle_impl.inc", "if (!touched[ord[p].i]) { rest = ord[p].a; break; }",
     "{ rest = ord[p].a; break; }"),
    ("roulette_reversed", "alns_oracle_impl.inc", "const int d_op = (ud * (w[0] + w[1]) < w[0]) ? 0 : 1;",
     "const int d_op = (ud * (w[0] + w[1]) < w[0]) ? 1 : 0;"),
    ("repair_weight_goes_to_destroy", "alns_oracle_impl.inc", "w[2 + r_op] = keep * w[2 + r_op] + prm->lambda * psi;",
     "w[r_op] = keep * w[r_op] + prm->lambda * psi;"),
    ("rejected_state_kept", "alns_oracle_impl.inc", "            memcpy(kidx, k_cur, (size_t)n * sizeof(int32_t));\n        }",
     "        }"),
    ("returns_current_not_best", "alns_oracle_impl.inc", "    memcpy(kidx, k_best, (size_t)n * sizeof(int32_t));\n    if (weights_out)",
     "    memcpy(kidx, k_cur, (size_t)n * sizeof(int32_t));\n    if (weights_out)"),
    ("reward_of_a_new_best", "alns_oracle_impl.inc", "psi = prm->sigma1;", "psi = prm->sigma2;"),
    ("guard_reversed", "alns_oracle_impl.inc", "(!prm->l2_guard || q2 <= q2_cur)", "(!prm->l2_guard || q2 >= q2_cur)"),
    ("impact_shift_dropped", "alns_oracle_impl.inc", "weight[j] = 1 + (sum >> shift);", "weight[j] = 1 + sum;"),
    ("impact_scale_exponent", "alns_oracle_impl.inc", "const double scale = ldexp(1.0, 24 - e);", "const double scale = ldexp(1.0, 23 - e);"),
    ("repair_error_skips_untouched_rows", "alns_oracle_impl.inc",
     "        if (!touched[i]) { REAL a = FABS(r[i]); if (a > out) out = a; }\n    for (int64_t p = colptr[j]; p < colptr[j + 1]; ++p) touched[rowidx[p]] = 0;\n    return out;",
     "        if (touched[i]) { REAL a = FABS(r[i]); if (a > out) out = a; }\n    for (int64_t p = colptr[j]; p < colptr[j + 1]; ++p) touched[rowidx[p]] = 0;\n    return out;"),
    ("random_repair_bit", "alns_oracle_impl.inc", "(uint64_t)pos) & 1) ? kc + 1 : kc - 1;", "(uint64_t)pos) & 2) ? kc + 1 : kc - 1;"),
    ("repair_at_an_end_of_D", "alns_oracle_impl.inc", "knew = has_lo ? kc - 1 : kc + 1;", "knew = kc;"),
    ("swap_ignores_scale", "swap_oracle_impl.inc",
     "    const REAL diff = D[kidx[i]] - D[kidx[j]];\n    const REAL Delta = sc * diff;\n    REAL out = (REAL)0;",
     "    const REAL diff = D[kidx[i]] - D[kidx[j]];\n    const REAL Delta = diff;\n    REAL out = (REAL)0;"),
    ("alns_scores_ignore_the_scale", "alns_oracle_impl.inc",
     "                REAL delta = SFX(delta_of)(D, kidx[j], k, sc);\n                out = rest;",
     "                REAL delta = SFX(delta_of)(D, kidx[j], k, (REAL)1);\n                out = rest;"),
    ("impact_ignores_the_scale", "alns_oracle_impl.inc", "const double a = fabs((double)sc * (double)cval[p]);",
     "const double a = fabs((double)cval[p]);"),
    ("repair_ignores_the_scale", "alns_oracle_impl.inc", "const REAL delta = SFX(delta_of)(D, kc, knew, sc);",
     "const REAL delta = SFX(delta_of)(D, kc, knew, (REAL)1);"),
    ("greedy_repair_scores_without_the_scale", "alns_oracle_impl.inc", "SFX(delta_of)(D, kc, kc - 1, sc));",
     "SFX(delta_of)(D, kc, kc - 1, (REAL)1));"),
    ("alns_start_residual_ignores_the_scale", "alns_oracle_impl.inc",
     "        r[i] = FMA(acc, sc, -b[i]);\n    }\n    REAL t_cur", "        r[i] = FMA(acc, (REAL)1, -b[i]);\n    }\n    REAL t_cur"),
    ("alns_local_search_applies_without_the_scale", "alns_oracle_impl.inc",
     "            const REAL delta = SFX(delta_of)(D, kidx[j], k, sc);\n            t = SFX(oracle_apply_move_csc)",
     "            const REAL delta = SFX(delta_of)(D, kidx[j], k, (REAL)1);\n            t = SFX(oracle_apply_move_csc)"),
    ("alns_local_search_takes_plateau_moves", "alns_oracle_impl.inc",
     "            if (c < 0 || !(s < t)) break;\n            const int64_t j = c / nd;",
     "            if (c < 0 || !(s <= t)) break;\n            const int64_t j = c / nd;"),
    ("alns_local_search_radius_ignored", "alns_oracle_impl.inc", "kidx, r, prm->ls_radius, scores);", "kidx, r, 0, scores);"),
    ("default_destroy_count_rounds_down", "alns_common.inc", "const int64_t c = (n * 5 + 999) / 1000;",
     "const int64_t c = (n * 5) / 1000;"),
    ("vanishing_error_threshold", "alns_oracle_impl.inc", "if (!(t >= 0x1p-900)) {", "if (!(t >= 0x1p-800)) {"),
    ("l2_cross_term_sign", "l2_oracle_impl.inc", "const REAL twog = (REAL)2 * g[j];", "const REAL twog = (REAL)-2 * g[j];"),
    ("l2_square_term_dropped", "l2_oracle_impl.inc", "dq[j * nd + k] = delta * FMA(delta, csq[j], twog);", "dq[j * nd + k] = delta * twog;"),
    ("l2_key_prefers_the_larger_change", "l2_oracle_impl.inc", "(scores[e] == s && dq[e] < q)", "(scores[e] == s && dq[e] > q)"),
    ("l2_guard_ignored", "l2_oracle_impl.inc", "if (rule == 2 && !(dq[e] <= (REAL)0)) continue;", "if (0) continue;"),
    ("l2_guard_drops_unchanged_norm", "l2_oracle_impl.inc", "if (rule == 2 && !(dq[e] <= (REAL)0)) continue;",
     "if (rule == 2 && !(dq[e] < (REAL)0)) continue;"),
    ("l2_changes_ignore_the_scale", "l2_oracle_impl.inc",
     "            const REAL delta = SFX(delta_of)(D, kidx[j], k, sc);\n            const REAL twog",
     "            const REAL delta = SFX(delta_of)(D, kidx[j], k, (REAL)1);\n            const REAL twog"),
    ("l2_column_sum_reads_the_wrong_row", "l2_oracle_impl.inc", "acc = FMA(cval[e], r[rowidx[e]], acc);",
     "acc = FMA(cval[e], r[e - colptr[j]], acc);"),
    ("l2_descent_takes_plateau_moves", "l2_oracle_impl.inc",
     "        if (c < 0 || !(s < t)) break;\n        const int64_t j = c / nd; const int32_t k = (int32_t)(c % nd);\n        const REAL delta = SFX(delta_of)(D, kidx[j], k, sc);\n        t = SFX(oracle_apply_move_csc)",
     "        if (c < 0 || !(s <= t)) break;\n        const int64_t j = c / nd; const int32_t k = (int32_t)(c % nd);\n        const REAL delta = SFX(delta_of)(D, kidx[j], k, sc);\n        t = SFX(oracle_apply_move_csc)"),
    ("l2_descent_scores_without_the_untouched_rows", "l2_oracle_impl.inc", "                        else v = FABS(r[i]);", "                        else v = (REAL)0;"),
]


def _build_mutant(tmp, fname, old, new):
    for f in os.listdir(ORACLE):
        if f.endswith((".c", ".inc")):
            shutil.copy(os.path.join(ORACLE, f), os.path.join(tmp, f))
    path = os.path.join(tmp, fname)
    src = open(path).read()
    assert src.count(old) == 1, f"the text to replace must occur exactly once in {fname}"
    open(path, "w").write(src.replace(old, new))
    lib = os.path.join(tmp, "liboracle_mutant.so")
    cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC", "-shared",
           "-o", lib, os.path.join(tmp, "dmmv_oracle.c"), "-lm"]
    if " fma " in open("/proc/cpuinfo").read().replace("\n", " "):
        cmd.insert(1, "-mfma")
    subprocess.check_call(cmd, cwd=tmp)
    return lib


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
@pytest.mark.parametrize("name,fname,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_the_pins_catch_a_planted_mistake(tmp_path, name, fname, old, new):
    lib = _build_mutant(str(tmp_path), fname, old, new)
    env = dict(os.environ, DMMV_ORACLE_LIB=lib)
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PIN_TESTS],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    assert run.returncode != 0, f"no pin noticed the mistake '{name}':\n{run.stdout[-2000:]}"


def test_the_unchanged_oracle_passes_in_the_same_harness(tmp_path):
    lib = _build_mutant(str(tmp_path), "dmmv_oracle.c", "#include <math.h>", "#include <math.h>")
    env = dict(os.environ, DMMV_ORACLE_LIB=lib)
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PIN_TESTS],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert run.returncode == 0, run.stdout[-2000:]

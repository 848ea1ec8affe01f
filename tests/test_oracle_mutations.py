"""The pins must notice a wrong oracle: each plausible mistake below is planted
in a copy of the C source (on the CPU, in a temporary directory), the copy is
compiled, and the pin tests are run against it; at least one must fail.  This
checks the pins, not the oracle: the shipped source is never modified."""
import importlib.util
import os
import shutil
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)

# (name, text in oracle/csp_oracle.c, replacement)
MUTATIONS = [
    ("scale_by_D_not_sqrtD", "const double inv_sqrt_d = 1.0 / sqrt((double)D);\n    for (int i = 0; i < O; ++i) {",
     "const double inv_sqrt_d = 1.0 / (double)D;\n    for (int i = 0; i < O; ++i) {"),
    ("causal_off_by_one", "const int n_vis = causal ? p + 1 : L;", "const int n_vis = causal ? p : L;"),
    ("window_starts_one_late", "const int p = L - O + i;                 /* absolute position of query i */",
     "const int p = L - O + i + 1 > L - 1 ? L - 1 : L - O + i + 1;"),
    ("n_added_after_max_subtraction", "double denom = n_score * exp(-m);\n        for (int j = 0; j < n_vis; ++j) denom",
     "double denom = n_score;\n        for (int j = 0; j < n_vis; ++j) denom"),
    ("n_dropped_when_scoring", "double denom = n_score * exp(-m);\n        for (int j = 0; j < n_vis; ++j) denom",
     "double denom = 0.0;\n        for (int j = 0; j < n_vis; ++j) denom"),
    ("self_and_cross_swapped", "if (mod[j] == mod[p]) a_self[j] += a;\n                else                  a_cross[j] += a;",
     "if (mod[j] != mod[p]) a_self[j] += a;\n                else                  a_cross[j] += a;"),
    ("recent_keys_ranked", "if (j < L - R) {\n                if (mod[j] == mod[p])", "if (j < L) {\n                if (mod[j] == mod[p])"),
    ("trim_one_too_many", "if (j < L - R) {\n                if (mod[j] == mod[p])", "if (j < L - R - 1) {\n                if (mod[j] == mod[p])"),
    ("mean_instead_of_sum_changes_nothing_but_sqrt", "const double a = exp(s[j] - m) / denom;\n            rs += a;",
     "const double a = sqrt(exp(s[j] - m) / denom);\n            rs += a;"),
    ("budget_ignores_recent", "const int K_sel = T - R;", "const int K_sel = T;"),
    ("ratio_gives_self_share", "int kc = (int)floor(cross_ratio * (double)K_sel);", "int kc = K_sel - (int)floor(cross_ratio * (double)K_sel);"),
    ("ratio_rounded_up", "int kc = (int)floor(cross_ratio * (double)K_sel);", "int kc = (int)ceil(cross_ratio * (double)K_sel);"),
    ("no_spill", "if (ks > n_s) { kc += ks - n_s; ks = n_s; }\n    if (kc > n_c) { ks += kc - n_c; kc = n_c; }",
     "if (ks > n_s) { ks = n_s; }\n    if (kc > n_c) { kc = n_c; }"),
    ("ties_prefer_higher_index", "return (x->idx > y->idx) - (x->idx < y->idx);", "return (x->idx < y->idx) - (x->idx > y->idx);"),
    ("smallest_instead_of_largest", "if (x->score > y->score) return -1;\n    if (x->score < y->score) return 1;",
     "if (x->score > y->score) return 1;\n    if (x->score < y->score) return -1;"),
    ("one_key_too_many", "for (int t = 0; t < K && t < c; ++t) mark[it[t].idx] = 1;", "for (int t = 0; t <= K && t < c; ++t) mark[it[t].idx] = 1;"),
    # (L < T instead of L <= T is not a mistake: at L == T the spill rule keeps everything too)
    ("early_out_one_too_generous", "if (L <= T) {                               /* identity */", "if (L <= T + 1) {"),
    ("candidates_ignore_window", "cand_s[j] = (uint8_t)has_q[mj];         /* some window query shares j's modality */",
     "cand_s[j] = 1;"),
    ("cross_candidates_same_as_self", "cand_c[j] = (uint8_t)has_q[1 - mj];     /* some window query has the other one */",
     "cand_c[j] = (uint8_t)has_q[mj];"),
    ("intersection_by_default", "const int in = combine == 0 ? (m_s[j] | m_c[j]) : (m_s[j] & m_c[j]);",
     "const int in = combine == 0 ? (m_s[j] & m_c[j]) : (m_s[j] & m_c[j]);"),
    ("recent_keys_forgotten", "for (int j = P; j < L; ++j) idx_out[kept++] = j;", "for (int j = P + 1; j < L; ++j) idx_out[kept++] = j;"),
    ("gather_wrong_row", "(const char*)src + (size_t)idx[t] * row_bytes, row_bytes);", "(const char*)src + (size_t)(idx[t] > 0 ? idx[t] - 1 : 0) * row_bytes, row_bytes);"),
    ("decode_n_after_max_subtraction", "double denom = n * exp(-m);\n    for (int t = 0; t < T; ++t) denom", "double denom = n;\n    for (int t = 0; t < T; ++t) denom"),
    ("decode_n_ignored", "double denom = n * exp(-m);\n    for (int t = 0; t < T; ++t) denom", "double denom = 0.0;\n    for (int t = 0; t < T; ++t) denom"),
    ("decode_unscaled_logits", "s[t] = dot * inv_sqrt_d;\n        if (s[t] > m) m = s[t];\n    }\n    for (int d = 0; d < D; ++d) out[d] = 0.0;",
     "s[t] = dot;\n        if (s[t] > m) m = s[t];\n    }\n    for (int d = 0; d < D; ++d) out[d] = 0.0;"),
    ("decode_uses_keys_as_values", "for (int d = 0; d < D; ++d) out[d] += p * vc[(size_t)t * D + d];", "for (int d = 0; d < D; ++d) out[d] += p * kc[(size_t)t * D + d];"),
    ("decode_skips_last_key", "for (int t = 0; t < T; ++t) {\n        const double p = exp(s[t] - m) / denom;", "for (int t = 0; t < T - 1; ++t) {\n        const double p = exp(s[t] - m) / denom;"),
]

# pin tests cheap enough to run against every mutant (name, kwargs for parametrised ones)
def _pins():
    import test_oracle_pins as P
    runs = []
    for seed in (0, 1, 3, 4):
        runs.append((P.test_scores_match_brute_force_tiny, dict(seed=seed)))
    for seed in range(8):
        runs.append((P.test_select_matches_brute_force_tiny, dict(seed=seed)))
    runs += [(P.test_exact_rational_example, {}), (P.test_scale_is_sqrt_head_dim, {}),
             (P.test_row_sums_closed_form, dict(n_score=1.0)), (P.test_row_sums_closed_form, dict(n_score=0.0)),
             (P.test_decode_equals_library_attention_with_virtual_zero_key, {}), (P.test_nsoftmax_shift_law, {}),
             (P.test_nsoftmax_undoes_sharpness_shift, {}), (P.test_full_budget_is_identity, dict(T_minus_L=0)),
             (P.test_budget_one_below_length_drops_exactly_one, {}), (P.test_zero_queries_closed_form_and_tie_rule, {}),
             (P.test_budget_rule_golden, {}), (P.test_gather_is_a_bit_copy, {}), (P.test_mixed_window_masks_overlap, {}),
             (P.test_counts_and_order_invariants, dict(ratio=0.5)), (P.test_visual_window_swaps_regions, {})]
    return runs


def _load_mutant(tmpdir, name, old, new):
    src = open(os.path.join(ROOT, "oracle", "csp_oracle.c")).read()
    assert src.count(old) == 1, f"mutation {name}: pattern occurs {src.count(old)} times"
    d = os.path.join(tmpdir, name)
    os.makedirs(d)
    with open(os.path.join(d, "csp_oracle.c"), "w") as f:
        f.write(src.replace(old, new))
    shutil.copy(os.path.join(ROOT, "oracle", "csp_oracle.py"), os.path.join(d, "csp_oracle.py"))
    spec = importlib.util.spec_from_file_location(f"csp_oracle_mut_{name}", os.path.join(d, "csp_oracle.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)      # _HERE inside it is the temporary directory: it compiles the mutant there
    mod.build(force=True)
    return mod


def _run_pins(mutant):
    """Runs the pins against `mutant` until one fails; returns its name (None: all passed)."""
    for fn, kw in _pins():
        try:
            fn(mutant, **kw)
        except BaseException as e:   # assertion, ValueError from a now-invalid call, pytest.fail, ...
            if isinstance(e, (KeyboardInterrupt, SystemExit)):
                raise
            return fn.__name__
    return None


# A mutant is wrong code on purpose, and wrong C code may also write out of bounds (one key too many
# overruns the caller's index buffer): every mutant therefore runs in a process of its own, where a
# crash is one more way of being noticed and cannot corrupt the heap of the test session.
_EXIT_NOTICED, _EXIT_UNNOTICED = 3, 0


def _child(tmpdir, index):
    name, old, new = MUTATIONS[index]
    sys.path.insert(0, HERE)
    sys.path.insert(0, ROOT)
    failed = _run_pins(_load_mutant(tmpdir, name, old, new))
    print(f"mutant {name}: {'noticed by ' + failed if failed else 'NOT noticed'}", flush=True)
    return _EXIT_NOTICED if failed else _EXIT_UNNOTICED


@pytest.mark.parametrize("index", range(len(MUTATIONS)), ids=[m[0] for m in MUTATIONS])
def test_pins_catch_planted_mistake(tmp_path, index):
    import subprocess
    res = subprocess.run([sys.executable, os.path.abspath(__file__), str(tmp_path), str(index)],
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    # exit 3: a pin failed; a signal or any other status: the mutant crashed (noticed as well)
    assert res.returncode != _EXIT_UNNOTICED, f"no pin noticed the planted mistake '{MUTATIONS[index][0]}'\n{res.stdout}"


def test_unmutated_source_passes_the_same_pins(tmp_path):
    sys.path.insert(0, HERE)
    src = open(os.path.join(ROOT, "oracle", "csp_oracle.c")).read()
    clean = _load_mutant(str(tmp_path), "clean", src[:40], src[:40])
    assert _run_pins(clean) is None


if __name__ == "__main__":
    sys.exit(_child(sys.argv[1], int(sys.argv[2])))

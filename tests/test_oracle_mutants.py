"""Do the pins bite?  Each case plants one plausible mistake in a copy of the oracle's C source
(a dropped term, a wrong sign or index, a non-strict comparison, a swapped tie-break), builds it,
and runs the oracle's pin tests against that build in a child process: at least one pin has to
fail.  CPU only; nothing here touches the HIP path or a GPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "spindle_oracle.c")

DEEP = ["tests/test_oracle_deep.py"]
SHALLOW = ["tests/test_oracle_shallow.py"]
DECODE = ["tests/test_oracle_decode.py"]
HELPERS = ["tests/test_oracle_deep.py::test_layer_ratio_pins", "tests/test_host_helpers.py"]
BUDGETS = ["tests/test_oracle_deep.py::test_layer_budget_pins"]       # the oracle's own pin, not the comparison with the library

# (name, text in the source, what it becomes, which occurrence, pin files)
MUTANTS = [
    ("softmax_sum_misses_the_query_position",
     "for (int a = 0; a <= p; ++a) Z += exp(s[a] - M);", "for (int a = 0; a < p; ++a) Z += exp(s[a] - M);", 0, DEEP),
    ("scale_dropped", "s[a] = dot * scale;", "s[a] = dot;", 0, DEEP),
    ("divisor_of_eq2_off_by_one", "v /= (double)(l - a);", "v /= (double)(l - a + 1);", 0, DEEP),
    ("group_sum_instead_of_mean", "out[a] /= (double)hn;", "out[a] /= 1.0;", 0, DEEP),
    ("window_sum_skips_first_query", "for (int b = 0; b < lw; ++b) {\n            const double *q",
     "for (int b = 1; b < lw; ++b) {\n            const double *q", 0, DEEP),
    ("weights_not_divided_by_the_row_sum", "acc[a] += exp(s[a] - M) / Z;", "acc[a] += exp(s[a] - M);", 0, DEEP),
    ("query_position_off_by_one", "int p = lc + b;                       /* position of this query */",
     "int p = lc + b - 1;", 0, DEEP),
    ("pool_ignores_the_first_position", "if (j >= 0 && j < n && x[j] > m) m = x[j];", "if (j >= 1 && j < n && x[j] > m) m = x[j];", 0, DEEP),
    ("pool_radius_one_too_wide", "int r = (P - 1) / 2;", "int r = (P + 1) / 2;", 0, DEEP),
    ("topk_ties_take_the_higher_index", "return (a > b) - (a < b);", "return (a < b) - (a > b);", 0, DEEP),
    ("window_positions_shifted", "kept[k + b] = lc + b;", "kept[k + b] = lc + b - 1;", 0, DEEP),
    ("magnitude_without_root", "m[a] = sqrt(ss);", "m[a] = ss;", 0, SHALLOW),
    ("cosine_of_zero_vector_is_one", "return den > 0.0 ? dot / den : 0.0;", "return den > 0.0 ? dot / den : 1.0;", 0, SHALLOW),
    ("cosine_denominator_uses_one_norm_twice", "double den = m[a] * m[b];", "double den = m[a] * m[a];", 0, SHALLOW),
    ("threshold_not_strict", "if (oracle_cos(X, m, d, a, b) > theta) {", "if (oracle_cos(X, m, d, a, b) >= theta) {", 0, SHALLOW),
    ("no_diagonal", "        SETBIT(G + (size_t)a * W, a);\n", "", 0, SHALLOW),
    ("adjacency_not_mirrored", "                SETBIT(G + (size_t)b * W, a);\n", "", 0, SHALLOW),
    ("row_spot_check_without_diagonal", "if (b == a || oracle_cos(X, m, d, a, b) > theta) SETBIT(row, b);",
     "if (oracle_cos(X, m, d, a, b) > theta) SETBIT(row, b);", 0, SHALLOW),
    ("references_numbered_from_one", "for (int b = 0; b < n; ++b) if (GETBIT(row, b)) ref[b] = nc;",
     "for (int b = 0; b < n; ++b) if (GETBIT(row, b)) ref[b] = nc + 1;", 0, SHALLOW),
    ("literal_loop_keeps_rows_of_removed_tokens", "if (GETBIT(row, a)) { for (int w = 0; w < W; ++w) ga[w] = 0; }",
     "if (0) { for (int w = 0; w < W; ++w) ga[w] = 0; }", 0, SHALLOW),
    ("incremental_loop_rereferences_removed_tokens", "if (alive[b] && GETBIT(row, b)) { ref[b] = nc; dying[nd++] = b; }",
     "if (GETBIT(row, b)) { ref[b] = nc; if (alive[b]) dying[nd++] = b; }", 0, SHALLOW),
    ("literal_loop_keeps_removed_columns", "ga[w] &= ~row[w];", "ga[w] &= ~0u;", 0, SHALLOW),
    ("incremental_loop_ties_take_the_higher_index",
     "if (alive[a] && deg[a] > bestdeg)", "if (alive[a] && deg[a] >= bestdeg)", 0, SHALLOW),
    ("incremental_loop_never_lowers_degrees", "if (alive[v]) deg[v]--;", "if (alive[v]) deg[v] -= 0;", 0, SHALLOW),
    ("cap_keeps_one_entry_too_many", "if (ref[a] < cap) continue;", "if (ref[a] <= cap) continue;", 0, SHALLOW),
    ("cap_ties_take_the_higher_entry", "if (c > bv) { bv = c; best = j; }", "if (c >= bv) { bv = c; best = j; }", 0, SHALLOW),
    ("codebook_not_normalised", "C[(size_t)c * d + t] = mm > 0.0 ? x[t] / mm : 0.0;", "C[(size_t)c * d + t] = x[t];", 0, SHALLOW),
    ("reconstruction_without_magnitude", "C[(size_t)ref[a] * d + t] * mag[a];", "C[(size_t)ref[a] * d + t];", 0, SHALLOW),
    ("decode_takes_the_last_suitable_entry", "if (cs > theta && cs > bv) { bv = cs; best = c; }",
     "if (cs > theta) { bv = cs; best = c; }", 0, DECODE),
    ("decode_ignores_the_entry_norm", "double den = mag[a] * cn[c];", "double den = mag[a];", 0, DECODE),
    ("decode_threshold_not_strict", "if (cs > theta && cs > bv)", "if (cs >= theta && cs > bv)", 0, DECODE),
    ("decode_new_entries_not_appended", "ref[rest[j]] = rr[j] < room ? nc + rr[j] : -1;",
     "ref[rest[j]] = rr[j] < room ? rr[j] : -1;", 0, DECODE),
    ("budget_second_case_as_printed", "r1 = 2.0 * rc - 1.0;", "r1 = 1.0 - 2.0 * rc;", 0, HELPERS),
    ("budget_first_case_without_beta", "r0 = 2.0 * rc - beta; r1 = beta;", "r0 = 2.0 * rc; r1 = beta;", 0, HELPERS),
    ("r1_inverted", "out[0] = kept / total;", "out[0] = total / kept;", 0, HELPERS),
    ("alpha_without_the_half", "double alpha = 0.5 * (1.0 + beta);", "double alpha = 1.0 + beta;", 0, HELPERS),
    ("r3_without_the_magnitude", "out[2] = (dh + (double)int_bit / key_bit + (double)mag_bit / key_bit) / dh;",
     "out[2] = (dh + (double)int_bit / key_bit) / dh;", 0, HELPERS),
    ("r3_magnitude_always_one_element", "out[2] = (dh + (double)int_bit / key_bit + (double)mag_bit / key_bit) / dh;",
     "out[2] = (dh + (double)int_bit / key_bit + 1.0) / dh;", 0, HELPERS),
    ("budget_rounded_to_nearest", "int k = (int)floor(rc[lam] * (double)(l - lw));",
     "int k = (int)floor(rc[lam] * (double)(l - lw) + 0.5);", 0, BUDGETS),
    ("budget_without_the_window", "budgets_out[lam] = lw + k;", "budgets_out[lam] = k;", 0, BUDGETS),
    ("budget_of_the_whole_length", "int k = (int)floor(rc[lam] * (double)(l - lw));",
     "int k = (int)floor(rc[lam] * (double)l);", 0, BUDGETS),
    ("budget_not_kept_at_zero", "if (k < 0) k = 0;", "", 0, BUDGETS),
]


def nth_replace(text, old, new, which):
    at = -1
    for _ in range(which + 1):
        at = text.find(old, at + 1)
        assert at >= 0, f"mutation site not found: {old!r}"
    return text[:at] + new + text[at + len(old):]


def run_pins(lib, files):
    env = dict(os.environ, SPINDLE_ORACLE_LIB=lib)
    return subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-m", "not gpu", "-p", "no:cacheprovider", *files],
                          cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)


def build(src_text, out_dir, name):
    c = os.path.join(out_dir, name + ".c")
    so = os.path.join(out_dir, name + ".so")
    with open(c, "w") as f:
        f.write(src_text)
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-w", "-o", so, c, "-lm"])
    return so


def test_unchanged_copy_passes_every_pin(tmp_path):
    # the control: the same procedure with no mistake planted must pass, or a failure below means nothing
    so = build(open(SRC).read(), str(tmp_path), "control")
    r = run_pins(so, DEEP + SHALLOW + DECODE + ["tests/test_host_helpers.py"])
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name,old,new,which,files", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_pin_fails(tmp_path, name, old, new, which, files):
    so = build(nth_replace(open(SRC).read(), old, new, which), str(tmp_path), name)
    r = run_pins(so, files)
    # 1 = a test failed.  Anything else (0: every pin passed; a crash) is not a pin doing its job.
    assert r.returncode == 1, f"{name}: pytest exit {r.returncode}\n{r.stdout[-1500:]}"

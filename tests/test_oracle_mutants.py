"""Are the pins strong enough?  Every entry below plants one plausible mistake (a dropped term, a
wrong index or sign, a skipped comparison) in a copy of the oracle's C source, on the CPU; the copy
is compiled and the pin tests run against it in a process of their own.  Each mutant has to make at
least one pin fail.  Nothing here touches the GPU path."""
import concurrent.futures as cf
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "recd_oracle.c")

# (name, text in the oracle, replacement, which occurrence)
MUTANTS = [
    ("half_subnormal_scale", "v = ldexp((double)man, -24);", "v = ldexp((double)man, -25);", 0),
    ("half_exponent_bias", "v = ldexp(1.0 + (double)man / 1024.0, exp - 15);",
     "v = ldexp(1.0 + (double)man / 1024.0, exp - 16);", 0),
    ("bf16_shift", "uint32_t bits = (uint32_t)h << 16;", "uint32_t bits = (uint32_t)h << 15;", 0),
    ("ikjt_prefix_match", "if (u_offsets[s + 1] - u_offsets[s] != len)\n                    continue;\n"
     "                const int64_t *cand",
     "if (u_offsets[s + 1] - u_offsets[s] < len)\n                    continue;\n"
     "                const int64_t *cand", 0),
    ("ikjt_search_across_features", "for (int64_t s = first_slot; s < U && found < 0; s++) {\n"
     "                if (u_offsets[s + 1]", "for (int64_t s = 0; s < U && found < 0; s++) {\n"
     "                if (u_offsets[s + 1]", 0),
    ("ikjt_inverse_global", "inverse[(int64_t)f * B + b] = (int32_t)(found - first_slot);",
     "inverse[(int64_t)f * B + b] = (int32_t)(found);", 0),
    ("grouped_first_feature_only", "for (int f = f0; f < f1 && same; f++) {", "for (int f = f0; f < f0 + 1 && same; f++) {", 0),
    ("grouped_slot_order", "const int64_t l = (int64_t)f * B + slot_row[k];", "const int64_t l = (int64_t)f * B + slot_row[n_slots - 1 - k];", 0),
    ("partial_overlap_shortest", "for (int64_t k = (last_len < len ? last_len : len); k >= 1 && overlap == 0; k--) {",
     "for (int64_t k = 1; k <= (last_len < len ? last_len : len) && overlap == 0; k++) {", 0),
    ("partial_overlap_any_predecessor", "if (b > 0 && U > first_slot && inverse[l - 1] == (int32_t)(U - 1 - first_slot)) {",
     "if (b > 0 && U > first_slot) {", 0),
    ("lookup_wrong_table", "o[d] += elem(tables[f], dtype, id * D + d);", "o[d] += elem(tables[0], dtype, id * D + d);", 0),
    ("lookup_transposed", "o[d] += elem(tables[f], dtype, id * D + d);", "o[d] += elem(tables[f], dtype, d * rows[f] + id);", 0),
    ("mean_divides_by_len_plus_one", "o[d] /= (double)len;", "o[d] /= (double)(len + 1);", 0),
    ("max_keeps_minimum", "o[d] = (j == offsets[l] || x > o[d]) ? x : o[d];", "o[d] = (j == offsets[l] || x < o[d]) ? x : o[d];", 0),
    ("weighted_builder_ignores_weights",
     "memcmp(u_weights + u_offsets[s], weights + at, sizeof(float) * len) == 0)", "1)", 0),
    ("weighted_lookup_drops_weight", "o[d] += (double)weights[j] * elem(tables[f], dtype, id * D + d);",
     "o[d] += elem(tables[f], dtype, id * D + d);", 0),
    ("group_sum_skips_offset", "o[d] += pooled[(feat_uoff[f] + k) * D + d];", "o[d] += pooled[(feat_uoff[group_off[g]] + k) * D + d];", 0),
    ("expand_local_index", "memcpy(out + ((int64_t)f * B + b) * D, pooled + (feat_uoff[f] + u) * D,",
     "memcpy(out + ((int64_t)f * B + b) * D, pooled + (u) * D,", 0),
    ("sequence_lookup_wrong_row", "emb[j * D + d] = elem(tables[f], dtype, id * D + d);",
     "emb[j * D + d] = elem(tables[f], dtype, j % rows[f] * D + d);", 0),
    ("jagged_expand_source_shift", "memcpy(out + (offsets[l] + t) * D, emb + (u_offsets[u] + t) * D, sizeof(double) * D);",
     "memcpy(out + (offsets[l] + t) * D, emb + (u_offsets[u] + len - 1 - t) * D, sizeof(double) * D);", 0),
    ("backward_step1_local_slot", "int64_t u = feat_uoff[f] + inverse[(int64_t)f * B + b];\n"
     "            const float *g", "int64_t u = inverse[(int64_t)f * B + b];\n            const float *g", 0),
    ("backward_step2_once_per_list", "G[k * D + d] += g_u[u * D + d];\n            }",
     "G[k * D + d] += (j == u_offsets[u]) ? g_u[u * D + d] : 0.0;\n            }", 0),
    ("backward_kjt_wrong_sample", "G[k * D + d] += (double)g[d];", "G[k * D + d] += (double)g[D - 1 - d];", 0),
    ("mean_backward_no_division", "G[k * D + d] += g_u[u * D + d] / len;", "G[k * D + d] += g_u[u * D + d];", 0),
    ("mean_backward_kjt_no_division", "G[k * D + d] += (double)grad_out[l * D + d] / len;",
     "G[k * D + d] += (double)grad_out[l * D + d];", 0),
    ("weighted_backward_drops_weight", "G[k * D + d] += (double)u_weights[j] * g_u[u * D + d];",
     "G[k * D + d] += g_u[u * D + d];", 0),
    ("weighted_backward_kjt_drops_weight", "G[k * D + d] += (double)weights[j] * (double)grad_out[l * D + d];",
     "G[k * D + d] += (double)grad_out[l * D + d];", 0),
    ("sequence_backward_step1_offset", "g_emb[(u_offsets[u] + t) * D + d] += (double)grad_out[(offsets[l] + t) * D + d];",
     "g_emb[(u_offsets[u] + t) * D + d] += (double)grad_out[(offsets[l] + len - 1 - t) * D + d];", 0),
    ("sequence_backward_kjt_sign", "G[k * D + d] += (double)grad_out[p * D + d];", "G[k * D + d] -= (double)grad_out[p * D + d];", 0),
    ("adagrad_sum_instead_of_mean", "double m = m_rows[r] + ss / (double)D;", "double m = m_rows[r] + ss;", 0),
    ("adagrad_eps_inside_root", "double denom = sqrt(m) + eps;", "double denom = sqrt(m + eps);", 0),
    ("adagrad_sign", "w_rows[r * D + d] - lr * grad_rows[r * D + d] / denom;", "w_rows[r * D + d] + lr * grad_rows[r * D + d] / denom;", 0),
    ("max_backward_last_wins", "if (best < 0 || tables[f][u_values[j] * D + d] > tables[f][u_values[best] * D + d])",
     "if (best < 0 || tables[f][u_values[j] * D + d] >= tables[f][u_values[best] * D + d])", 0),
    ("max_backward_kjt_minimum", "if (best < 0 || tables[f][values[j] * D + d] > tables[f][values[best] * D + d])",
     "if (best < 0 || tables[f][values[j] * D + d] < tables[f][values[best] * D + d])", 0),
    ("first_rows_keeps_last", "if (first_row[feat_uoff[f] + k] < 0)\n", "if (1)\n", 0),
    ("first_rows_local_row", "first_row[feat_uoff[f] + k] = (int64_t)f * B + b;", "first_row[feat_uoff[f] + k] = b;", 0),
    ("run_crosses_feature", "if (b > 0 && inverse[l - 1] == k)\n                continue; /* the row continues",
     "if (l > 0 && inverse[l - 1] == k)\n                continue; /* the row continues", 0),
    ("run_first_flag_always", "run_first[R] = !seen;", "run_first[R] = 1;", 0),
    ("run_list_local", "const int64_t u = feat_uoff[f] + k;\n            run_row[R] = l;",
     "const int64_t u = k;\n            run_row[R] = l;", 0),
    ("touched_rows_unsorted", "qsort(tmp, n, sizeof(int64_t), cmp_i64);\n    int64_t r = 0;",
     "int64_t r = 0;", 0),
]


def _run_mutant(tmp, name, old, new, which):
    text = open(SRC).read()
    at = -1
    for _ in range(which + 1):
        at = text.find(old, at + 1)
        assert at >= 0, f"{name}: the oracle no longer contains the text this mutant replaces"
    text = text[:at] + new + text[at + len(old):]
    c_path, so_path = os.path.join(tmp, name + ".c"), os.path.join(tmp, name + ".so")
    open(c_path, "w").write(text)
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", c_path, "-o", so_path,
                           "-lm"])
    env = dict(os.environ, RECD_ORACLE_LIB=so_path)
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider", "--timeout", "120"], cwd=ROOT, env=env, capture_output=True,
                       text=True, timeout=300)
    return name, r.returncode, r.stdout[-400:]


def test_every_mutant_fails_a_pin(tmp_path):
    with cf.ThreadPoolExecutor(max_workers=6) as ex:
        results = list(ex.map(lambda m: _run_mutant(str(tmp_path), *m), MUTANTS))
    survivors = [(n, out) for n, rc, out in results if rc == 0]
    assert not survivors, "mutants that no pin notices: " + ", ".join(n for n, _ in survivors)
    # a crash of the mutated oracle (signal) also counts as noticed; a collection error does not
    broken = [(n, rc, out) for n, rc, out in results if rc not in (1,) and rc >= 0 and rc != 0]
    assert not broken, f"pin run did not end in test failures: {broken}"


def test_unmutated_copy_passes(tmp_path):
    name, rc, out = _run_mutant(str(tmp_path), "identity", "int oracle_check_kjt(", "int oracle_check_kjt(", 0)
    assert rc == 0, out

"""The pins must notice plausible mistakes.

Each case plants ONE mistake in a copy of the oracle's C source (on the CPU), builds it,
and runs the pin suite against that build in a child process: the suite has to fail.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "pikv_oracle.c")

MUTANTS = {
    "softmax_scale_dropped": ("s[i] = scale * dot;", "s[i] = dot;"),
    "gqa_head_map_modulo": ("const int hk = h / G;", "const int hk = h % Hkv;"),
    "router_weight_transposed": ("load_elem(W_r, (int64_t)j * E + e, dtype)",
                                 "load_elem(W_r, ((int64_t)e * d_r + j) % ((int64_t)d_r * E), dtype)"),
    "router_penalty_dropped": ("if (bias) acc += (double)bias[e];", ""),
    "router_tie_break_reversed": ("return (x->e > y->e) - (x->e < y->e);",
                                  "return (x->e < y->e) - (x->e > y->e);"),
    "lse_gate_ignored_in_output": ("const double w = g * Z[j] * exp(m[j] - M) / norm;",
                                   "const double w = Z[j] * exp(m[j] - M) / norm;"),
    "local_gates_not_renormalised": ("const double gh = (gsel ? (double)gsel[j] : 1.0) / norm;",
                                     "const double gh = (gsel ? (double)gsel[j] : 1.0);"),
    "shard_max_not_subtracted_consistently": ("s[i] = exp(s[i] - m[j]);", "s[i] = exp(s[i]);"),
    "value_rows_read_from_keys": ("entry_vector(Vs, hk, i, stride_h, stride_s, D, rank, U_V, V_bias, dtype, kv);",
                                  "entry_vector(Ks, hk, i, stride_h, stride_s, D, rank, U_V, V_bias, dtype, kv);"),
    "decoder_transposed": ("load_elem(U, ((int64_t)hk * rank + c) * D + d, dtype)",
                           "load_elem(U, ((int64_t)hk * D + d) * rank + c, dtype)"),
    "utility_decay_dropped": ("u[i] = (float)(decay * (double)u[i] + a);",
                              "u[i] = (float)((double)u[i] + a);"),
    "utility_counts_every_head": ("if (topk_idx[(int64_t)row * k + j] == e)\n                                a +=",
                                  "if (1)\n                                a +="),
    "evict_tie_break_reversed": ("return (x->slot > y->slot) - (x->slot < y->slot);",
                                 "return (x->slot < y->slot) - (x->slot > y->slot);"),
    "evict_keeps_lowest": ("if (x->u > y->u) return -1;\n    if (x->u < y->u) return 1;\n    return (x->slot",
                           "if (x->u > y->u) return 1;\n    if (x->u < y->u) return -1;\n    return (x->slot"),
    "append_keeps_old_utility": ("utility[be * S + slot] = 0.0f;", ""),
    "load_penalty_sign_flipped": ("bias[e] = (float)(-coef * ((double)load[e] - mean));",
                                  "bias[e] = (float)(coef * ((double)load[e] - mean));"),
    "load_penalty_not_centred": ("mean /= (double)E;", "mean = 0.0;"),
    "miss_penalty_without_log": ("bias[e] = (float)(-coef * log(1.0 + (double)miss[e]));",
                                 "bias[e] = (float)(-coef * (double)miss[e]);"),
    "encoder_transposed": ("load_elem(W_enc, ((int64_t)h * rank + c) * D + d, dtype)",
                           "load_elem(W_enc, (((int64_t)h * D + d) * rank + c) % ((int64_t)Hkv * rank * D), dtype)"),
    "lru_sign_flipped": ("u = (policy == 2) ? -r : fmaf(lambda, (float)freq[x], -r);",
                         "u = (policy == 2) ? r : fmaf(lambda, (float)freq[x], -r);"),
    "lru_plus_rounded_twice": ("fmaf(lambda, (float)freq[x], -r);", "(float)(lambda * (float)freq[x]) - r;"),
    "lru_plus_frequency_sign": ("fmaf(lambda, (float)freq[x], -r);", "fmaf(-lambda, (float)freq[x], -r);"),
    "window_off_by_one": ("u = (now - birth[x] < window) ? 1.0f : 0.0f;",
                          "u = (now - birth[x] <= window) ? 1.0f : 0.0f;"),
    "protect_compare_reversed": ("if (protect > 0 && now - birth[x] < protect) u = INFINITY;",
                                 "if (protect > 0 && now - birth[x] > protect) u = INFINITY;"),
    "access_counts_equal_as_above": ("if (mass[be * S + i] > threshold) {", "if (mass[be * S + i] >= threshold) {"),
    "access_frequency_not_counted": ("freq[be * S + i] += 1;", ""),
    "access_touches_dead_slots": ("for (int i = 0; i < n_valid[be]; ++i) {\n            if (mass",
                                  "for (int i = 0; i < S; ++i) {\n            if (mass"),
    "stamp_ignores_freed_slot": ("if (reuse_cnt && reuse_cnt[be] > 0) slot = reuse_idx[be * max_evict];\n            if (slot < 0 || slot >= S || n_valid[be] >= S) return -3;\n            birth",
                                 "if (slot < 0 || slot >= S || n_valid[be] >= S) return -3;\n            birth"),
    "stamp_keeps_old_frequency": ("freq[be * S + slot] = 0;", ""),
    "policy_compact_skips_hole_test": ("if (g < cnt && gone[g] == i) { ++g; continue; }", "if (g < cnt && gone[g] == i) { ++g; }"),
    "round_robin_ignores_k_stride": ("(int32_t)(((step + r) * k + j) % E);", "(int32_t)(((step + r) + j) % E);"),
    "entropy_penalty_not_centred": ("bias[e] = (float)(-coef * (he - h_avg));", "bias[e] = (float)(-coef * he);"),
    "entropy_penalty_sign_flipped": ("bias[e] = (float)(-coef * (he - h_avg));", "bias[e] = (float)(coef * (he - h_avg));"),
    "entropy_of_counts_not_shares": ("const double pe = total > 0.0 ? (double)load[e] / total : 0.0;\n            const double he",
                                     "const double pe = (double)load[e];\n            const double he"),
    "value_bias_added_to_keys_too": ("entry_vector(Ks, hk, i, stride_h, stride_s, D, rank, U_K, NULL, dtype, kv);",
                                     "entry_vector(Ks, hk, i, stride_h, stride_s, D, rank, U_K, V_bias, dtype, kv);"),
    "value_bias_wrong_head": ("acc += load_elem(U_bias, (int64_t)hk * D + d, dtype);",
                              "acc += load_elem(U_bias, (int64_t)d, dtype);"),
    "empty_shard_counted_in_local_norm": ("if (Z[j] > 0.0) norm += gsel ? (double)gsel[j] : 1.0;",
                                          "norm += gsel ? (double)gsel[j] : 1.0;"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_fail_on_planted_mistake(name, tmp_path):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) == 1, "mutation anchor must match exactly once: %r" % old
    src = tmp_path / "mutant.c"
    src.write_text(text.replace(old, new))
    lib = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-w",
                           "-o", str(lib), str(src), "-lm"])
    env = dict(os.environ, PIKV_ORACLE_LIB=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    assert r.returncode != 0, "pins did not notice mutant %s" % name
    assert b"failed" in r.stdout, r.stdout[-2000:].decode()

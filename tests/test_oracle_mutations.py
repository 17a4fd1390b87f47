"""Checks that the oracle's pins have teeth: each plausible mistake below is
planted in a copy of the oracle source (on the CPU), and the pin tests must
fail against that copy."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "rec_oracle.c")

MUTATIONS = {
    "fc_transposed_weight": ("W[(int64_t)o * n_in + i]", "W[(int64_t)i * n_out + o]"),
    "fc_dropped_bias": ("apply_act(acc + (double)bias[o], act)", "apply_act(acc, act)"),
    "fc_bf16_ignored": ("if (bf16_operands) {", "if (0) {"),
    "sigmoid_sign": ("1.0 / (1.0 + exp(-z))", "1.0 / (1.0 + exp(z))"),
    "relu_dropped": ("z > 0.0 ? z : 0.0", "z"),
    "sls_bag_order_sample_major": ("const int64_t bag = (int64_t)t * B + b;", "const int64_t bag = (int64_t)b * T + t;"),
    "sls_drops_last_lookup": ("p < off[bag + 1]; ++p", "p < off[bag + 1] - 1; ++p"),
    "sls_row_stride": ("(int64_t)indices[p] * D", "(int64_t)indices[p] * (D - 1)"),
    "interact_upper_order": ("for (int32_t i = 1; i < V; ++i)\n            for (int32_t j = 0; j < i; ++j) {",
                             "for (int32_t j = 0; j < V; ++j)\n            for (int32_t i = j + 1; i < V; ++i) {"),
    "interact_includes_diagonal": ("for (int32_t j = 0; j < i; ++j) {", "for (int32_t j = 0; j <= i && p < D + V * (V - 1) / 2; ++j) {"),
    "interact_slot0_not_copied": ("o[d] = v[d];", "o[d] = v[D + d];"),
    "bf16_truncates": ("u += 0x7fffu + lsb;", "u += 0;"),
    "validate_upper_bound_off_by_one": (">= rows[t])", "> rows[t])"),
    "validate_ignores_negative": ("indices[pos] < 0 || ", ""),
    "offsets_inclusive": ("off[i + 1] = off[i] + lengths[i];", "off[i + 1] = off[i] + lengths[i + 1 < n_bags ? i + 1 : i];"),
    "model_top_uses_relu_last": ("ORC_ACT_RELU, ORC_ACT_SIGMOID, inter", "ORC_ACT_RELU, ORC_ACT_RELU, inter"),
    "model_sls_into_slot0": ("vecs + D, (int64_t)V * D, D, NULL, NULL", "vecs, (int64_t)V * D, D, NULL, NULL"),
    "split_drops_tail": ("(n - s < Bsz) ? n - s : Bsz", "Bsz"),
    "service_drops_remainder": ("if (n % B) s += t[n % B];", ""),
    "fifo_ignores_queue": ("(i > 0 && prev_finish > arrival[i]) ? prev_finish : arrival[i]", "arrival[i]"),
    "fifo_latency_excludes_wait": ("latency[i] = prev_finish - arrival[i];", "latency[i] = service[i];"),
    "percentile_off_by_one": ("(int64_t)ceil(p * (double)n) - 1;", "(int64_t)ceil(p * (double)n);"),
    "max_qps_returns_infeasible_end": ("    free(lat);\n    return lo;", "    free(lat);\n    return hi;"),
    "concat_embeddings_overwrite_dense": ("orc_sls(tables, T, D, indices, off, B, cat + X, Wc, D, NULL, NULL);",
                                          "orc_sls(tables, T, D, indices, off, B, cat, Wc, D, NULL, NULL);"),
    "concat_table_stride": ("orc_sls(tables, T, D, indices, off, B, cat + X, Wc, D, NULL, NULL);",
                            "orc_sls(tables, T, D, indices, off, B, cat + X, Wc, 1, NULL, NULL);"),
    "concat_dense_dropped": ("cat[b * Wc + f] = dense[(int64_t)b * X + f];", "cat[b * Wc + f] = 0.0f;"),
    "concat_dense_transposed": ("cat[b * Wc + f] = dense[(int64_t)b * X + f];",
                                "cat[b * Wc + f] = dense[((int64_t)f * B + b) % ((int64_t)B * X)];"),
    "two_tier_threshold_exclusive": ("if (m >= tau) {", "if (m > tau) {"),
    "two_tier_busiest_worker": ("if (free_at[j] < free_at[w]) w = j;", "if (free_at[j] > free_at[w]) w = j;"),
    "two_tier_done_is_last_request": ("if (free_at[w] > done) done = free_at[w];", "done = free_at[w];"),
    "two_tier_accelerator_never_queues": ("const double start = gpu_free > arrival[i] ? gpu_free : arrival[i];",
                                          "const double start = arrival[i];"),
    "two_tier_request_before_arrival": ("const double start = free_at[w] > arrival[i] ? free_at[w] : arrival[i];",
                                        "const double start = free_at[w];"),
    "two_tier_full_batches_only": ("const int64_t b = (m - first < B) ? m - first : B;", "const int64_t b = B;"),
    "hill_climb_stops_on_ties": ("qps[i + 1] >= qps[i]", "qps[i + 1] > qps[i]"),
    "hill_climb_global_max": ("while (i + 1 < n_candidates && qps[i + 1] >= qps[i]) ++i;",
                              "for (int64_t j = 1; j < n_candidates; ++j) if (qps[j] > qps[i]) i = j;"),
}


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_pins_catch_planted_mistake(name, tmp_path):
    old, new = MUTATIONS[name]
    src = open(SRC).read()
    assert src.count(old) >= 1, f"mutation target not found: {old!r}"
    mutated = tmp_path / "mut.c"
    mutated.write_text(src.replace(old, new, 1))
    lib = tmp_path / "libmut.so"
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-o", str(lib), str(mutated), "-lm"])
    env = dict(os.environ, REC_ORACLE_LIB=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        os.path.join(ROOT, "tests", "test_oracle_sched_pins.py")],
                       env=env, cwd=ROOT, capture_output=True, text=True, timeout=300)
    assert r.returncode != 0, f"pins did not notice mutation {name}"
    assert "failed" in r.stdout

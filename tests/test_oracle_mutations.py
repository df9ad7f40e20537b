"""The pins must notice plausible mistakes in the oracle.

Each case below plants ONE mistake in a private copy of `oracle/e4q_oracle.c` (on the CPU, in a
temporary directory), rebuilds it and re-runs `test_oracle_pins.py` against that copy: the run
must fail.  The test that compares the C oracle with its NumPy twin is left out of those runs,
because agreement between two implementations of one reading is not a pin.
"""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

KMEANS_MUTANTS = {
    "sixteen_grid_intervals": ("float step = (hi - lo) / 15.0f;", "float step = (hi - lo) / 16.0f;"),
    "ties_take_the_higher_index": ("if (dk < bd) { bd = dk; best = k; }", "if (dk <= bd) { bd = dk; best = k; }"),
    "one_round_short": ("for (int it = 0; it < lloyd_iters; ++it) {", "for (int it = 1; it < lloyd_iters; ++it) {"),
    "empty_cluster_moves_to_zero": ("if (cnt[k] > 0) c[k] = (float)(sum[k] / (double)cnt[k]);",
                                    "c[k] = cnt[k] > 0 ? (float)(sum[k] / (double)cnt[k]) : 0.0f;"),
    "sum_instead_of_mean": ("c[k] = (float)(sum[k] / (double)cnt[k]);", "c[k] = (float)(sum[k]);"),
    "indices_from_unrounded_centres": ("unsigned q0 = (unsigned)nearest_centre(x[2 * b], ch);",
                                       "unsigned q0 = (unsigned)nearest_centre(x[2 * b], c);"),
    "index_nibbles_swapped": ("out[b] = (uint8_t)(q0 | (q1 << 4));\n            }\n        } else {",
                              "out[b] = (uint8_t)(q1 | (q0 << 4));\n            }\n        } else {"),
    "small_rows_clustered": ("if (dim <= K) {", "if (dim <= 0) {"),
    "squared_distance_sign": ("float dk = fabsf(x - c[k]);", "float dk = x - c[k];"),
    "binary16_bits_read_as_integers": ("for (int k = 0; k < d; ++k) dst[k] = e4q_oracle_f16_to_f32(src[k]);",
                                       "for (int k = 0; k < d; ++k) dst[k] = (float)src[k];"),
    "binary16_rows_at_binary32_pitch": ("const uint16_t *src = (const uint16_t *)table + row * row_stride;",
                                        "const uint16_t *src = (const uint16_t *)table + 2 * row * row_stride;"),
    "binary16_row_starts_one_late": ("dst[k] = e4q_oracle_f16_to_f32(src[k]);", "dst[k] = e4q_oracle_f16_to_f32(src[k ? k : 1]);"),
}

SLS_MUTANTS = {
    "nibbles_swapped": ("unsigned q = (k & 1) ? (byte >> 4) : (byte & 0xfu);", "unsigned q = (k & 1) ? (byte & 0xfu) : (byte >> 4);"),
    "bag_starts_one_late": ("for (int64_t i = offsets[b]; i < offsets[b + 1]; ++i) {", "for (int64_t i = offsets[b] + 1; i < offsets[b + 1]; ++i) {"),
    "bag_runs_one_over": ("i < offsets[b + 1]; ++i) {", "i <= offsets[b + 1]; ++i) {"),
    "right_to_left": ("for (int64_t i = offsets[b]; i < offsets[b + 1]; ++i) {", "for (int64_t i = offsets[b + 1] - 1; i >= offsets[b]; --i) {"),
    "bias_dropped": ("e4q_oracle_f16_to_f32(bias_f16[r]));", "0.0f);"),
    "last_row_rejected": ("if (r < 0 || r >= rows) continue;", "if (r < 0 || r >= rows - 1) continue;"),
    "scale_of_wrong_row": ("e4q_oracle_f16_to_f32(scale_f16[r])", "e4q_oracle_f16_to_f32(scale_f16[b])"),
}

MUTANTS = {
    "sixteen_levels": ("return (float)((1 << nbits) - 1); }", "return (float)(1 << nbits); }"),
    "tie_moves_lower_bound": ("if (loss_l < loss_r) {", "if (loss_l <= loss_r) {"),
    "later_equal_loss_wins": ("if (loss_r < best.loss) {", "if (loss_r <= best.loss) {"),
    "upper_bound_moves_up": ("float next_max = cur_max - stepsize;", "float next_max = cur_max + stepsize;"),
    "round_half_up": ("float q = rintf(t);", "float q = floorf(t + 0.5f);"),
    "truncate": ("float q = rintf(t);", "float q = truncf(t);"),
    "strided_sum_tree": ("s[i] = s[2 * i] + s[2 * i + 1];", "s[i] = s[i] + s[i + m / 2];"),
    "nibbles_swapped": ("byte |= q << (s * nbits);", "byte |= q << ((per - 1 - s) * nbits);"),
    "search_ignores_fp16_storage": ("*scale = round_through_f16(scale32);", "*scale = scale32;"),
    "no_upper_clamp": ("if (q > qmax) q = qmax;", ""),
    "no_lower_clamp": ("if (q < 0.0f) q = 0.0f;", "if (q < 0.0f) q = -q;"),
    "step_off_by_one": ("float stepsize = (hi0 - lo0) / (float)n_bins;\n    float cur_min",
                        "float stepsize = (hi0 - lo0) / (float)(n_bins - 1);\n    float cur_min"),
    "floor_trip_count": ("double t = ceil(br - br * 0x1p-22);", "double t = floor(br);"),
    "start_not_a_candidate": ("best.loss = range_loss(x, d, lo0, hi0, qmax, work);", "best.loss = INFINITY;"),
    "literal_bookkeeping_by_default": ("if (!literal_alg1) { best.xmax = cur_max; best.j = j; }",
                                       "if (literal_alg1) { best.xmax = cur_max; best.j = j; }"),
    "dequantize_nibbles_swapped": ("unsigned q = (byte >> ((k % per) * nbits)) & mask;",
                                   "unsigned q = (byte >> ((per - 1 - k % per) * nbits)) & mask;"),
    "bias_is_not_xmin": ("*bias_f16 = e4q_oracle_f32_to_f16(lo);", "*bias_f16 = e4q_oracle_f32_to_f16(hi);"),
    "error_not_squared": ("work[k] = e * e;", "work[k] = fabsf(e);"),
    "f16_ties_away": ("if (rem > 0x1000u || (rem == 0x1000u && (h & 1u)))", "if (rem >= 0x1000u)"),
    "binary16_bits_read_as_integers": ("for (int k = 0; k < d; ++k) dst[k] = e4q_oracle_f16_to_f32(src[k]);",
                                       "for (int k = 0; k < d; ++k) dst[k] = (float)src[k];"),
    "binary16_rows_at_binary32_pitch": ("const uint16_t *src = (const uint16_t *)table + row * row_stride;",
                                        "const uint16_t *src = (const uint16_t *)table + 2 * row * row_stride;"),
    "zero_minimum_keeps_its_sign": ("    lo0 = lo0 + 0.0f;\n    hi0 = hi0 + 0.0f;\n    greedy_result best", "    greedy_result best"),
}


def _run_pins(oracle_parent, test_file="test_oracle_pins.py"):
    env = dict(os.environ)
    if oracle_parent:
        env["E4Q_TEST_ORACLE_PARENT"] = oracle_parent
    return subprocess.run(
        [sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", test_file), "-x", "-q",
         "-k", "not numpy_twin", "-p", "no:cacheprovider"],
        cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_planted_mistake(name, tmp_path):
    old, new = MUTANTS[name]
    dst = tmp_path / "oracle"
    dst.mkdir()
    for f in ("__init__.py", "numpy_twin.py", "e4q_oracle.c", "e4q_oracle_kmeans.c", "e4q_oracle_sls.c"):
        shutil.copy(os.path.join(ROOT, "oracle", f), dst / f)
    src = (dst / "e4q_oracle.c").read_text()
    assert src.count(old) >= 1, f"mutation site for {name} no longer exists in the oracle"
    (dst / "e4q_oracle.c").write_text(src.replace(old, new))
    res = _run_pins(str(tmp_path))
    assert res.returncode != 0, f"pins did not notice mutant '{name}':\n{res.stdout[-2000:]}"
    assert "failed" in res.stdout or "error" in res.stdout.lower()


@pytest.mark.parametrize("name", sorted(KMEANS_MUTANTS))
def test_kmeans_pins_catch_planted_mistake(name, tmp_path):
    old, new = KMEANS_MUTANTS[name]
    dst = tmp_path / "oracle"
    dst.mkdir()
    for f in ("__init__.py", "numpy_twin.py", "e4q_oracle.c", "e4q_oracle_kmeans.c", "e4q_oracle_sls.c"):
        shutil.copy(os.path.join(ROOT, "oracle", f), dst / f)
    src = (dst / "e4q_oracle_kmeans.c").read_text()
    assert src.count(old) >= 1, f"mutation site for {name} no longer exists in the oracle"
    (dst / "e4q_oracle_kmeans.c").write_text(src.replace(old, new, 1))
    res = _run_pins(str(tmp_path), "test_oracle_kmeans_pins.py")
    assert res.returncode != 0, f"pins did not notice mutant '{name}':\n{res.stdout[-2000:]}"


@pytest.mark.parametrize("name", sorted(SLS_MUTANTS))
def test_sls_pins_catch_planted_mistake(name, tmp_path):
    old, new = SLS_MUTANTS[name]
    dst = tmp_path / "oracle"
    dst.mkdir()
    for f in ("__init__.py", "numpy_twin.py", "e4q_oracle.c", "e4q_oracle_kmeans.c", "e4q_oracle_sls.c"):
        shutil.copy(os.path.join(ROOT, "oracle", f), dst / f)
    src = (dst / "e4q_oracle_sls.c").read_text()
    assert src.count(old) >= 1, f"mutation site for {name} no longer exists in the oracle"
    (dst / "e4q_oracle_sls.c").write_text(src.replace(old, new, 1))
    res = _run_pins(str(tmp_path), "test_oracle_sls_pins.py")
    assert res.returncode != 0, f"pins did not notice mutant '{name}':\n{res.stdout[-2000:]}"

"""Are the oracle's pins sharp?  Each case plants ONE plausible mistake in a copy of the
oracle's source (a dropped mask, a wrong sign, a swapped index, a tie broken the other way),
builds it, and runs the pin tests against that copy in a child process: the named pin must
fail.  The mistakes live in a temporary directory on the CPU; the product and the real oracle
are untouched."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "kvcrush_oracle.cpp")

# (name, text in the oracle, replacement, pin test expected to notice)
MUTATIONS = [
    ("no causal mask", "for (int j = 0; j <= i; ++j) c[j] += p[j] / L;",
     "for (int j = 0; j < S; ++j) c[j] += (j <= i ? p[j] : p[i]) / L;",
     "tests/test_oracle_scores.py::test_brute_force_full_matrix"),
    ("no 1/sqrt(D)", "const double inv_sqrt_d = scale != 0.0 ? scale : 1.0 / std::sqrt((double)D);\n  for (int i = row_begin",
     "const double inv_sqrt_d = scale != 0.0 ? scale : 1.0;\n  for (int i = row_begin",
     "tests/test_oracle_scores.py::test_against_library_softmax"),
    ("row sums instead of column sums", "c[j] += p[j] / L;", "c[i] += p[j] / L;",
     "tests/test_oracle_scores.py::test_uniform_attention_closed_form"),
    ("unnormalised probabilities", "c[j] += p[j] / L;", "c[j] += p[j];",
     "tests/test_oracle_scores.py::test_column_sums_total_the_number_of_rows"),
    ("window starts one row early", "const int row_begin = (obs_window == 0 || obs_window >= S) ? 0 : S - obs_window;",
     "const int row_begin = (obs_window == 0 || obs_window >= S) ? 0 : S - obs_window - 1;",
     "tests/test_oracle_scores.py::test_window_matches_brute_force_and_library"),
    ("ties to the higher index", "[v](int a, int b) { return v[a] > v[b]; }",
     "[v](int a, int b) { return v[a] > v[b] || (v[a] == v[b] && a > b); }",
     "tests/test_oracle_select.py::test_topk_tie_straddling_threshold"),
    ("alternating anchor starts with one", "if (r & 1) a[r / 64] |= 1ull << (r % 64);",
     "if (!(r & 1)) a[r / 64] |= 1ull << (r % 64);",
     "tests/test_oracle_select.py::test_anchor_modes"),
    ("majority not strict", "if (2 * cnt > N) a[r / 64]", "if (2 * cnt >= N) a[r / 64]",
     "tests/test_oracle_select.py::test_mean_anchor_strict_majority_over_discarded_only"),
    ("bucket cuts rounded up", "const long long lo = j * N / Br, hi = (j + 1) * N / Br;",
     "const long long lo = (j * N + Br - 1) / Br, hi = ((j + 1) * N + Br - 1) / Br;",
     "tests/test_oracle_select.py::test_hand_worked_examples"),
    ("medoid cost inverted", "? (n - cnt[r]) : cnt[r];", "? cnt[r] : (n - cnt[r]);",
     "tests/test_oracle_select.py::test_group_matches_pairwise_hamming_brute_force"),
    ("importance summed in double", "float acc = 0.0f;\n        for (int r = 0; r < Hs; ++r) acc = acc + mid[(size_t)r * Sm + u];\n        imp[u] = acc;",
     "double acc = 0.0;\n        for (int r = 0; r < Hs; ++r) acc = acc + mid[(size_t)r * Sm + u];\n        imp[u] = (float)acc;",
     "tests/test_oracle_select.py::test_importance_sum_is_sequential_fp32"),
    ("important tokens grouped too", "if (!is_important[t]) disc.push_back(t);", "disc.push_back(t);",
     "tests/test_oracle_select.py::test_select_matches_brute_force"),
    ("protected ends shifted", "const bool prot = t < n_sink || t >= S - n_recent;\n      const int u = t - n_sink;",
     "const bool prot = t < n_sink || t > S - n_recent;\n      const int u = t - n_sink;",
     "tests/test_oracle_select.py::test_protected_ends_match_brute_force_on_the_middle"),
    ("page vector interleaved the other way", "const int pos = j * Hs + r;", "const int pos = r * unit + j;",
     "tests/test_oracle_select.py::test_unit_level_hand_worked_example"),
    ("append adds to the new slot", "(j == S - 1 ? 0.0 : (double)row[j])", "((double)row[j])",
     "tests/test_oracle_decode.py::test_append_is_one_library_softmax_row"),
    ("append ignores the caller's scale", "const double inv_sqrt_d = scale != 0.0 ? scale : 1.0 / std::sqrt((double)D);\n  std::vector<double> logit(S), add(S);",
     "const double inv_sqrt_d = 1.0 / std::sqrt((double)D);\n  std::vector<double> logit(S), add(S);",
     "tests/test_oracle_decode.py::test_append_with_a_caller_scale_is_the_library_softmax_at_that_scale"),
    ("gather ignores the head", "const size_t src = (((size_t)b * Hkv + h) * cap_src + t) * row;",
     "const size_t src = (((size_t)b * Hkv + 0) * cap_src + t) * row;",
     "tests/test_oracle_decode.py::test_compact_cache_is_a_strided_gather"),
    ("max pool off centre", "for (int u = t - half; u <= t + half; ++u)", "for (int u = t - half + 1; u <= t + half; ++u)",
     "tests/test_oracle_scores.py::test_maxpool_matches_library"),
]


@pytest.mark.parametrize("name,old,new,pin", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(tmp_path, name, old, new, pin):
    src = open(SRC).read()
    assert src.count(old) >= 1, f"the oracle no longer contains the text this case mutates: {old!r}"
    mutated = tmp_path / "mutant.cpp"
    mutated.write_text(src.replace(old, new, 1))
    lib = tmp_path / "libmutant.so"
    subprocess.run(["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC", "-o",
                    str(lib), str(mutated)], check=True)
    env = dict(os.environ, KVCRUSH_ORACLE_LIB_FOR_MUTATION_TEST=str(lib))
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", pin], cwd=ROOT,
                         env=env, capture_output=True, text=True)
    assert run.returncode == 1, f"pin {pin} did not notice '{name}':\n{run.stdout[-2000:]}"
    assert "failed" in run.stdout


def test_unmutated_oracle_passes_the_same_pins():
    pins = sorted({m[3] for m in MUTATIONS})
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *pins], cwd=ROOT,
                         capture_output=True, text=True)
    assert run.returncode == 0, run.stdout[-2000:]

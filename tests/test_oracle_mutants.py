"""Are the pins sharp?  Plausible mistakes are planted in COPIES of the oracle source (on the
CPU, never in the GPU path); each mutant is compiled and the oracle's pin tests are run
against it in a subprocess.  Every mutant must be caught by at least one pin."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "combo_ref.cpp")
PIN_FILES = ["tests/test_oracle_pins.py", "tests/test_oracle_pooled.py", "tests/test_oracle_dynamic.py",
             "tests/test_oracle_divergence.py"]

# (name, text to replace, replacement): each is one wrong token of the kind that slips in
MUTANTS = [
    ("dropped_first_peer", "for (int32_t j = 0; j < R; ++j) acc = acc + X[(size_t)pl[j]",
     "for (int32_t j = 1; j < R; ++j) acc = acc + X[(size_t)pl[j]"),
    ("scale_by_R_not_R_plus_1", "const float inv = 1.0f / (float)(R + 1);", "const float inv = 1.0f / (float)(R);"),
    ("self_left_out", "float acc = X[(size_t)w * (size_t)ld + c];\n                    for (int32_t j = 0; j < R; ++j) acc",
     "float acc = 0.0f;\n                    for (int32_t j = 0; j < R; ++j) acc"),
    ("table_axes_transposed",
     "const int32_t* pl = peers + ((size_t)w * (size_t)S + (size_t)s) * (size_t)R;\n            int64_t lo = seg_lo(P, S, s), hi = seg_hi(P, S, s);\n            if (lo < col0) lo = col0;\n            if (hi > col0 + ncols) hi = col0 + ncols;\n            float den = 0.0f;",
     "const int32_t* pl = peers + ((size_t)s * (size_t)N + (size_t)w) * (size_t)R;\n            int64_t lo = seg_lo(P, S, s), hi = seg_hi(P, S, s);\n            if (lo < col0) lo = col0;\n            if (hi > col0 + ncols) hi = col0 + ncols;\n            float den = 0.0f;"),
    ("remainder_dropped", "return (s == S - 1) ? P : (int64_t)(s + 1) * seg_len(P, S);",
     "return (int64_t)(s + 1) * seg_len(P, S);"),
    ("hash_counters_swapped", "h = absorb(h, w);\n    h = absorb(h, s);", "h = absorb(h, s);\n    h = absorb(h, w);"),
    ("reduce_uses_low_bits", "return (uint32_t)(((h >> 32) * (uint64_t)m) >> 32);",
     "return (uint32_t)(((h & 0xFFFFFFFFull) * (uint64_t)m) >> 32);"),
    ("skip_self_off_by_one", "= c + (c >= w ? 1 : 0);", "= c + (c > w ? 1 : 0);"),
    ("shuffle_span_not_shrinking", "const int32_t r = j + (int32_t)reduce(h, (uint32_t)(M - j));\n                const int32_t t = a[(size_t)j];",
     "const int32_t r = (int32_t)reduce(h, (uint32_t)M);\n                const int32_t t = a[(size_t)j];"),
    ("weighted_den_without_self", "den = d[w];\n                for (int32_t j = 0; j < R; ++j) den = den + d[pl[j]];",
     "den = 0.0f;\n                for (int32_t j = 0; j < R; ++j) den = den + d[pl[j]];"),
    ("weighted_wrong_weight", "const float term = d[pl[j]] * X[(size_t)pl[j] * (size_t)ld + c];\n                        num = num + term;\n                    }\n                    Y[(size_t)w * (size_t)ld + c] = num / den;",
     "const float term = d[w] * X[(size_t)pl[j] * (size_t)ld + c];\n                        num = num + term;\n                    }\n                    Y[(size_t)w * (size_t)ld + c] = num / den;"),
    ("sgd_sign", "X[k] = X[k] - step;", "X[k] = X[k] + step;"),
    ("multi_step_only_last_gradient", "const float* Gk = G + (size_t)k * (size_t)N * (size_t)ld;",
     "const float* Gk = G + (size_t)(tau - 1) * (size_t)N * (size_t)ld;"),
    ("pooled_no_duplicate_check", "for (int32_t k = 0; k < j; ++k) taken = taken || picks[k] == queue[pos];",
     "for (int32_t k = 0; k < 0; ++k) taken = taken || picks[k] == queue[pos];"),
    ("pooled_refills_every_segment", "if (queue.empty()) {", "if (queue.empty() || j == 0) {"),
    ("dynamic_newcomer_keeps_own", "if (status[w] == 1) terms.push_back(w);", "if (status[w] != 0) terms.push_back(w);"),
    ("dynamic_asks_newcomers", "if (v != w && status[v] == 1) cand.push_back(v);", "if (v != w && status[v] != 0) cand.push_back(v);"),
    ("dynamic_offline_aggregates", "if (status[w] != 0)\n                for (int32_t j = 0; j < R; ++j)\n                    if (pl[j] >= 0) terms.push_back(pl[j]);",
     "for (int32_t j = 0; j < R; ++j)\n                    if (pl[j] >= 0) terms.push_back(pl[j]);"),
    ("divergence_unweighted_mean", "num += (d ? (long double)d[w] : 1.0L) * (long double)X[(size_t)w * (size_t)ld + (size_t)e];\n        const long double mean = num / den;",
     "num += (long double)X[(size_t)w * (size_t)ld + (size_t)e];\n        const long double mean = num / (long double)N;"),
    ("window_ignores_offset", "const size_t c = (size_t)(e - col0);\n                if (!d) {", "const size_t c = (size_t)(e);\n                if (!d) {"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_is_caught(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for {name} not found exactly once"
    mutant_src = tmp_path / "combo_ref_mutant.cpp"
    mutant_src.write_text(text.replace(old, new))
    lib = tmp_path / "libcombo_ref_mutant.so"
    subprocess.run(["g++", "-std=c++17", "-O1", "-ffp-contract=off", "-fPIC", "-shared", "-o", str(lib),
                    str(mutant_src)], check=True)
    out = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          "--oracle-lib", str(lib)] + PIN_FILES,
                         cwd=ROOT, capture_output=True, text=True, timeout=300)
    # a failed pin or a crash (some mutants write out of bounds) both count as caught
    assert out.returncode != 0, f"mutant {name} passed every pin:\n{out.stdout[-2000:]}"


def test_the_same_route_passes_with_an_unmodified_copy(tmp_path):
    """The control: a copy of the oracle as it stands, built and loaded the same way, passes
    every pin, so a non-zero exit above means a pin failed and not that the run went wrong."""
    lib = tmp_path / "libcombo_ref_copy.so"
    subprocess.run(["g++", "-std=c++17", "-O1", "-ffp-contract=off", "-fPIC", "-shared", "-o", str(lib), SRC],
                   check=True)
    out = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          "--oracle-lib", str(lib)] + PIN_FILES,
                         cwd=ROOT, capture_output=True, text=True, timeout=600)
    assert out.returncode == 0, out.stdout[-2000:] + out.stderr[-1000:]

"""Mutation check of the oracle's pins (CPU only).

Each case plants ONE plausible mistake in a copy of oracle/oracle.cpp (a text substitution),
compiles the copy, and runs the named pins of tests/test_oracle_pins.py against it in a child
process (the oracle's loader takes the library to load from ORACLE_LIBRARY).  The pins must fail:
a mistake of that kind in the real oracle would not go unnoticed.  The unmodified source must
pass the same pins, so a pin that fails for an unrelated reason does not count as a kill.
Nothing here touches the HIP path; the mistakes are planted in the CPU checker only.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

from oracle import build as oracle_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "oracle.cpp")
PINS = os.path.join(ROOT, "tests", "test_oracle_pins.py")

# (name, [(old text, new text, occurrences expected)], -k expression of the pins that must fail)
MUTANTS = [
    ("accumulate_subtracts",
     [("acc[i] = g[i] + eps[i];", "acc[i] = g[i] - eps[i];", 1)],
     "accumulate"),
    ("accumulate_truncates",
     [("acc[i] = g[i] + eps[i];",
       "{ double s_ = (double)g[i] + (double)eps[i]; float f_ = (float)s_; "
       "if (std::isfinite(f_) && std::fabs((double)f_) > std::fabs(s_)) "
       "f_ = std::nextafterf(f_, 0.0f); acc[i] = f_; }", 1)],
     "accumulate"),
    ("accumulate_flushes_denormals",
     [("acc[i] = g[i] + eps[i];",
       "{ float f_ = g[i] + eps[i]; acc[i] = std::fabs(f_) < 1.17549435e-38f ? 0.0f * f_ : f_; }", 1)],
     "accumulate"),
    ("nudge_factors_swapped",
     [("if (round < 3) thres = 0.5 * thres;", "if (round < 3) thres = 1.5 * thres;", 1),
      ("if (round < 3) thres = 1.5 * thres;\n    } else {", "if (round < 3) thres = 0.5 * thres;\n    } else {", 1)],
     "walk_on_level_vectors or uniform_grid"),
    ("compare_not_strict",
     [("(std::fabs(acc[i]) > t32) ? 1 : 0", "(std::fabs(acc[i]) >= t32) ? 1 : 0", 1),
      ("if (std::fabs(acc[i]) > t32) {", "if (std::fabs(acc[i]) >= t32) {", 1)],
     "strict"),
    ("lower_band_edge_exclusive",
     [("if (3 * est < 2 * k) {", "if (3 * est <= 2 * k) {", 1)],
     "walk_on_level_vectors"),
    ("upper_band_edge_exclusive",
     [("} else if (3 * est > 4 * k) {", "} else if (3 * est >= 4 * k) {", 1)],
     "walk_on_level_vectors"),
    ("three_evaluations",
     [("for (int round = 0; round <= 3; ++round) {\n    t32", "for (int round = 0; round <= 2; ++round) {\n    t32", 1)],
     "walk_on_level_vectors or uniform_grid"),
    ("mean_dropped_from_threshold",
     [("res->thres0 = res->mean + res->std * res->z;", "res->thres0 = res->std * res->z;", 1)],
     "walk_on_level_vectors or threshold_includes_the_mean"),
    ("std_divisor_ignores_ddof",
     [("std::sqrt(m2 / (double)(d - ddof))", "std::sqrt(m2 / (double)d)", 1)],
     "moments"),
    ("mean_of_absolute_values",
     [("for (int64_t i = 0; i < d; ++i) s += (double)acc[i];",
       "for (int64_t i = 0; i < d; ++i) s += std::fabs((double)acc[i]);", 1)],
     "moments"),
    ("one_sided_tail_by_default",
     [("const double q = (double)k / (tail_div * (double)d);", "const double q = (double)k / (double)d;", 1)],
     "needs_one_evaluation"),
    ("quantile_without_sqrt2",
     [("return 0.5 * std::erfc(z / std::sqrt(2.0));", "return 0.5 * std::erfc(z);", 1)],
     "norm_isf"),
    ("topk_ties_prefer_higher_index",
     [("(uint64_t)(0xFFFFFFFFu - (uint32_t)i);", "(uint64_t)(uint32_t)i;", 1),
      ("0xFFFFFFFFu - (uint32_t)(order[(size_t)j] & 0xFFFFFFFFu);",
       "(uint32_t)(order[(size_t)j] & 0xFFFFFFFFu);", 1)],
     "brute_force"),
    ("topk_keeps_one_too_few",
     [("std::nth_element(order.begin(), order.begin() + (k - 1), order.end(), std::greater<uint64_t>());\n"
       "  const uint64_t kth = order[(size_t)(k - 1)];",
       "std::nth_element(order.begin(), order.begin() + (k - 1), order.end(), std::greater<uint64_t>());\n"
       "  const uint64_t kth = order[(size_t)(k - 1)]; order[(size_t)(k - 1)] = order[(size_t)(d - 1)];", 1)],
     "brute_force"),
    ("topk_on_signed_values",
     [("inline uint32_t mag_key(float x) { return bits_of(x) & 0x7FFFFFFFu; }",
       "inline uint32_t mag_key(float x) { return bits_of(x) ^ 0x80000000u; }", 1)],
     "brute_force"),
    ("residual_keeps_selected_entries",
     [("    val[j] = acc[i];\n    eps_out[i] = 0.0f;", "    val[j] = acc[i];", 1)],
     "residual_identity"),
    ("sqnorm_of_absolute_values",
     [("s += (double)x[i] * (double)x[i];", "s += std::fabs((double)x[i]);", 1)],
     "randk"),
    ("dgck_keep_is_strict",
     [("if (mag_key(acc[i]) >= Ts) kept.push_back((uint32_t)i);",
       "if (mag_key(acc[i]) > Ts) kept.push_back((uint32_t)i);", 1)],
     "dgck"),
    ("dgck_rank_in_sample_rounds_down",
     [("const int64_t ks = (k * m + d - 1) / d;", "const int64_t ks = std::max<int64_t>(1, (k * m) / d);", 1)],
     "dgck"),
    ("scatter_add_overwrites",
     [("dense[pi[j]] = dense[pi[j]] + pv[j];", "dense[pi[j]] = pv[j];", 1)],
     "scatter_add"),
    ("scatter_add_takes_the_workers_backwards",
     [("for (int32_t p = 0; p < num_lists; ++p) {\n    const uint32_t* pi",
       "for (int32_t p = num_lists - 1; p >= 0; --p) {\n    const uint32_t* pi", 1)],
     "scatter_add"),
    ("scatter_add_scales_every_pair",
     [("dense[pi[j]] = dense[pi[j]] + pv[j];", "dense[pi[j]] = dense[pi[j]] + pv[j] * scale;", 1),
      ("dense[i] = dense[i] * scale;", "dense[i] = dense[i];", 1)],
     "scatter_add"),
    ("scatter_add_sums_in_fp64",
     [("for (int64_t i = 0; i < d; ++i) dense[i] = 0.0f;\n  // the sum over",
       "std::vector<double> wide((size_t)d, 0.0);\n  // the sum over", 1),
      ("dense[pi[j]] = dense[pi[j]] + pv[j];", "wide[pi[j]] += (double)pv[j];", 1),
      ("dense[i] = dense[i] * scale;", "dense[i] = (float)wide[(size_t)i] * scale;", 1)],
     "scatter_add"),
    ("segment_indices_stay_local",
     [("sidx[j] += (uint32_t)a;", "sidx[j] += 0u;", 1)],
     "segmented"),
]


def run_pins(library, expr):
    env = dict(os.environ)
    if library:
        env["ORACLE_LIBRARY"] = library
    else:
        env.pop("ORACLE_LIBRARY", None)
    return subprocess.run([sys.executable, "-m", "pytest", PINS, "-x", "-q", "-p", "no:cacheprovider",
                           "-k", expr], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                          stderr=subprocess.STDOUT, text=True, timeout=600)


def build_and_run(job):
    name, edits, expr, folder = job
    if name is None:                       # the unmodified source against every pin used below
        return run_pins(None, expr)
    text = open(SRC).read()
    for old, new, times in edits:
        assert text.count(old) == times, (name, old, text.count(old))
        text = text.replace(old, new)
    src = os.path.join(folder, f"oracle_{name}.cpp")
    with open(src, "w") as f:
        f.write(text)
    lib = oracle_build.build(src=src, out=os.path.join(folder, f"liboracle_{name}.so"))
    return run_pins(lib, expr)


@pytest.fixture(scope="module")
def outcomes(tmp_path_factory):
    """All the child processes at once, a few at a time (they are independent)."""
    folder = str(tmp_path_factory.mktemp("mutants"))
    every = " or ".join(sorted({f"({m[2]})" for m in MUTANTS}))
    jobs = [(None, None, every, folder)] + [(n, e, x, folder) for n, e, x in MUTANTS]
    with ThreadPoolExecutor(max_workers=6) as pool:
        done = list(pool.map(build_and_run, jobs))
    return {job[0]: out for job, out in zip(jobs, done)}


def test_unmodified_oracle_passes_every_pin_used_below(outcomes):
    out = outcomes[None]
    assert out.returncode == 0, out.stdout[-2000:]


@pytest.mark.parametrize("name,expr", [(m[0], m[2]) for m in MUTANTS], ids=[m[0] for m in MUTANTS])
def test_pins_fail_on_a_planted_mistake(name, expr, outcomes):
    out = outcomes[name]
    assert out.returncode == 1, f"mutant {name} survived the pins `{expr}`:\n{out.stdout[-1500:]}"
    assert "failed" in out.stdout

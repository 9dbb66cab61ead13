"""GPU parity of the flat calls against the CPU oracle: sizes that span several tiles and a
ragged tail, the degenerate inputs of both selectors, both buffer modes."""
import numpy as np
import pytest
import torch

from gpu_harness import FlatGpu, assert_pairs_match, check_flat, same_bits
from oracle import oracle as O
from paper_1911_08772_amd import sparsify as S
from paper_1911_08772_amd import synth

pytestmark = pytest.mark.gpu

SIZES = [1, 2, 3, 5, 63, 64, 65, 255, 1000, 4095, 4096, 4097, 8195, 12288, 100_003, 269_722]


def ks_for(d):
    return sorted({1, max(1, d // 1000), max(1, d // 10), max(1, d // 2), d})


@pytest.mark.parametrize("inplace", [False, True])
@pytest.mark.parametrize("selector", ["gaussiank", "topk"])
def test_sizes_and_densities(selector, inplace):
    for d in SIZES:
        g = synth.normal(d, 101, d, 0.01)
        eps = synth.normal(d, 102, d, 0.003)
        gpu = FlatGpu(d, cap=d, inplace=inplace)
        for k in ks_for(d):
            gpu.set_residual(eps)
            check_flat(selector, gpu, g, eps, k, what=f"{selector} d={d} k={k} inplace={inplace}")


def special_vectors(d, rng):
    out = {}
    out["small_ints"] = rng.integers(-3, 4, d).astype(np.float32)          # heavy ties, zeros
    v = rng.standard_normal(d).astype(np.float32)
    v[rng.integers(0, d, d // 3)] = np.float32(1.5)
    v[rng.integers(0, d, d // 3)] = np.float32(-1.5)
    out["planted_pm_ties"] = v
    w = (rng.integers(-4, 5, d) * np.float32(1e-45)).astype(np.float32)    # denormals, -0
    w[::7] = np.float32(-0.0)
    out["denormals"] = w
    out["zeros"] = np.zeros(d, np.float32)
    out["constant"] = np.full(d, 0.375, np.float32)
    u = rng.standard_normal(d).astype(np.float32)
    u[rng.integers(0, d, 5)] = np.float32(np.inf)
    u[rng.integers(0, d, 5)] = np.float32(-np.inf)
    out["infs"] = u
    n = rng.standard_normal(d).astype(np.float32)
    n[rng.integers(0, d, 3)] = np.float32(np.nan)
    out["nans"] = n
    big = (rng.standard_normal(d) * 1e30).astype(np.float32)
    out["huge"] = big
    return out


@pytest.mark.parametrize("d", [777, 4096, 20_011])
def test_topk_ties_and_special_values(d):
    rng = np.random.default_rng(d)
    zero = np.zeros(d, np.float32)
    gpu = FlatGpu(d, cap=d)
    for name, acc in special_vectors(d, rng).items():
        for k in sorted({1, 2, d // 7, d // 3, d // 2, d - 1, d}):
            gpu.set_residual(zero)
            check_flat("topk", gpu, acc, zero, k, what=f"topk {name} d={d} k={k}")


@pytest.mark.parametrize("inplace", [False, True])
def test_topk_ranked_ties_across_tile_groups(inplace):
    """Hundreds of tiles (several groups of 64), keys drawn from a handful of values: the k-th key
    is shared by thousands of entries and only the lowest-index ones are kept."""
    d = 1_000_003
    rng = np.random.default_rng(2024)
    zero = np.zeros(d, np.float32)
    vecs = {"small_ints": rng.integers(-3, 4, d).astype(np.float32),
            "two_exponents": (rng.integers(1, 5, d) * np.float32(0.5)).astype(np.float32),
            "constant": np.full(d, -2.5, np.float32)}
    late = np.zeros(d, np.float32)           # every tie of the k-th key sits in the last tiles
    late[d - 5000:] = 1.0
    late[:100] = 2.0
    vecs["ties_at_the_end"] = late
    gpu = FlatGpu(d, cap=d, inplace=inplace)
    for name, acc in vecs.items():
        for k in (1, 1000, d // 7, d // 2, d - 1):
            for tc in (1, 0):
                gpu.set_residual(zero)
                check_flat("topk", gpu, acc, zero, k, what=f"topk {name} k={k} tc={tc} inplace={inplace}",
                           tile_chunks=tc)


@pytest.mark.parametrize("d", [777, 20_011])
def test_gaussiank_special_values(d):
    rng = np.random.default_rng(d + 1)
    zero = np.zeros(d, np.float32)
    gpu = FlatGpu(d, cap=d)
    for name, acc in special_vectors(d, rng).items():
        for k in sorted({1, d // 100 + 1, d // 3}):
            for kw in ({}, {"tail_div": 1.0}, {"ddof": 0}):
                gpu.set_residual(zero)
                check_flat("gaussiank", gpu, acc, zero, k, what=f"gk {name} d={d} k={k} {kw}", **kw)


def test_gaussiank_multi_round_walks_and_overflow():
    # level vectors drive the threshold walk through x1.5 / x0.5 sequences (counts known exactly)
    d, k = 200_000, 90
    zero = np.zeros(d, np.float32)
    gpu = FlatGpu(d, cap=4 * k)
    for levels, small in [([(100, 10.0), (400, 1.0)], 2.0 ** -12), ([(180, 2.0)], 0.3125),
                          ([(60, 2.0)], 0.3125), ([(121, 2.0)], 0.3125), ([(59, 2.0)], 0.3125)]:
        x = np.full(d, small, np.float32)
        x[1::2] = -small
        pos = 0
        for cnt, mag in levels:
            x[pos:pos + cnt] = mag
            x[pos + 1:pos + cnt:2] = -mag
            pos += cnt
        gpu.set_residual(zero)
        check_flat("gaussiank", gpu, x, zero, k, what=f"levels {levels}")
    # heavy tails: several rounds; and a capacity too small for the final count
    x = synth.student_t3(d, 55, 0, 1e-3)
    for cap in (4 * k, 10):
        gpu = FlatGpu(d, cap=cap)
        gpu.set_residual(zero)
        check_flat("gaussiank", gpu, x, zero, k, what=f"student cap={cap}")
    res = S.decode_results(gpu.b.result)[0]
    assert res["flags"] & S.F_OVERFLOW and res["nnz"] == 0


@pytest.mark.parametrize("tile_chunks", [1, 3, 16])
@pytest.mark.parametrize("selector", ["gaussiank", "topk"])
def test_results_do_not_depend_on_the_tiling(selector, tile_chunks):
    for d in (5, 4097, 70_001, 1_000_003):
        g = synth.student_t3(d, 103, d, 1e-3)
        eps = synth.normal(d, 104, d, 0.003)
        gpu = FlatGpu(d, cap=d)
        for k in sorted({1, max(1, d // 1000), max(1, d // 20)}):
            gpu.set_residual(eps)
            check_flat(selector, gpu, g, eps, k, what=f"{selector} d={d} k={k} tc={tile_chunks}",
                       tile_chunks=tile_chunks)


def test_large_mean_keeps_moment_accuracy():
    # mean/std = 1e4: a one-pass raw-moment sum would lose the variance; the shifted sums do not
    d, k = 300_000, 300
    g = (100.0 + 0.01 * synth.normal(d, 77, 0, 1.0).astype(np.float64)).astype(np.float32)
    zero = np.zeros(d, np.float32)
    gpu = FlatGpu(d, cap=d)
    check_flat("gaussiank", gpu, g, zero, k, what="large mean")


@pytest.mark.parametrize("selector", ["gaussiank", "topk"])
def test_cfg1_error_feedback_chain(selector):
    """ResNet-20-sized vector: single shot, then 10 error-feedback iterations, fresh g each."""
    wl = synth.workload("cfg1_resnet20")
    gpu = FlatGpu(wl.d, cap=max(4 * wl.k, 1024))
    eps = np.zeros(wl.d, np.float32)
    for step in range(wl.steps + 1):
        eps = check_flat(selector, gpu, wl.grad(step), eps, wl.k, what=f"cfg1 {selector} step {step}")


def test_run_to_run_reproducibility():
    """Same inputs, repeated calls: identical result records, identical pair lists in identical
    (ascending index) order, identical residuals; every selector, separate accumulator and in
    place, the usual tilings and a forced one-chunk tiling that nearly fills the group tables."""
    wl = synth.workload("cfg1_resnet20")
    g = wl.grad(0)
    eps = synth.normal(wl.d, 9, 9, 0.002)
    g[1000:1400] = np.float32(0.25)    # many keys equal to the k-th key: ties ranked by index
    g[5000:5400:2] = np.float32(-0.25)
    eps[1000:1400] = 0
    eps[5000:5400] = 0
    for selector, inplace, kw in (("gaussiank", False, {}), ("gaussiank", True, {}),
                                  ("topk", False, {}), ("topk", True, {}), ("dgck", False, {}),
                                  ("topk", True, {"tile_chunks": 1}), ("topk", False, {"tile_chunks": 1})):
        d = wl.d if not kw else 16_000_000   # 3907 one-chunk tiles in 62 groups: the tables hold 4096
        gg = g if not kw else np.resize(g, d)
        ee = eps if not kw else np.resize(eps, d)
        k = wl.k if not kw else 16_000
        gpu = FlatGpu(d, cap=4 * k, inplace=inplace)
        ref = None
        for rep in range(20 if not kw else 4):
            gpu.set_residual(ee)
            got = gpu.step(selector, gg, k, **kw)
            now = (got["res"].tobytes(), got["eps"].tobytes(), got["idx"].tobytes(), got["val"].tobytes())
            if ref is None:
                ref = now
            assert now == ref, (selector, inplace, kw, rep)
        assert np.all(np.diff(got["idx"].astype(np.int64)) > 0), (selector, inplace, kw)
        if selector == "topk":
            assert int(got["res"]["topk_ties_taken"]) >= 1


def test_stream_argument_and_trace():
    wl = synth.workload("cfg1_resnet20")
    g = wl.grad(0)
    gpu = FlatGpu(wl.d, cap=4 * wl.k)
    side = torch.cuda.Stream()
    tr = S.Trace()
    b = gpu.b
    gpu.grad.copy_(torch.from_numpy(g))
    torch.cuda.synchronize()
    for fn, n_stage in ((S.sparsify_gaussiank, 3), (S.sparsify_topk, 7), (S.sparsify_dgck, 11)):
        b.residual.zero_()
        torch.cuda.synchronize()
        fn(wl.d, wl.k, gpu.grad, b.residual, b.acc, b.out_idx, b.out_val, gpu.cap, b.result,
           b.workspace, b.workspace_nbytes, trace=tr, stream=side)
        side.synchronize()
        stages = tr.stages()
        assert len(stages) == n_stage and all(ms >= 0 for _, ms in stages), stages
        res = S.decode_results(b.result)[0]
        assert res["nnz"] > 0
        idx_o, val_o, eps_o, _ = (O.gaussiank(g, wl.k, cap=gpu.cap) if fn is S.sparsify_gaussiank
                                  else O.topk(g, wl.k) if fn is S.sparsify_topk else O.dgck(g, wl.k))
        assert same_bits(b.residual.cpu().numpy(), eps_o)

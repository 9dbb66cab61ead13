"""GPU parity of the layer-wise call: ragged, misaligned and tiny segments, k_l = 1, segments
that overflow their output range, invalid layouts, and the 54-segment ResNet-50-sized workload."""
import numpy as np
import pytest
import torch

from gpu_harness import SegGpu, check_segmented, progress, same_bits
from oracle import oracle as O
from paper_1911_08772_amd import sparsify as S
from paper_1911_08772_amd import synth

pytestmark = pytest.mark.gpu


def layout(sizes, rho_den=100, cap_mult=4):
    sizes = np.asarray(sizes, np.int64)
    seg_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    seg_k = np.maximum(1, (sizes + rho_den - 1) // rho_den).astype(np.int64)
    caps = np.maximum(cap_mult * seg_k, 16).astype(np.int64)
    return seg_off, seg_k, caps


def seg_grad(seg_off, seed, step, sigmas):
    g = np.empty(int(seg_off[-1]), np.float32)
    for l in range(len(sigmas)):
        a, b = int(seg_off[l]), int(seg_off[l + 1])
        synth.normal(b - a, seed, step, float(sigmas[l]), g[a:b], index0=a)
    return g


SMALL_LAYOUTS = [
    [64, 1, 1000, 37, 4096, 5000, 3],
    [1],
    [4096, 4096, 4096],
    [4095, 4097, 1, 1, 1, 8191, 2],
    [3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37, 41, 43, 47, 53, 59, 61, 67, 71, 73] * 15,
    [100_000, 7, 250_001, 64],
    # segments of 74, 1, 171, exactly 64 and 65 tiles: several groups of 64 tiles per segment
    [300_000, 5, 700_001, 4096 * 64, 4096 * 64 + 1],
]


@pytest.mark.parametrize("inplace", [False, True])
@pytest.mark.parametrize("mode", [0, 1])
def test_small_layouts(mode, inplace):
    for n, sizes in enumerate(SMALL_LAYOUTS):
        seg_off, seg_k, caps = layout(sizes)
        sig = 10.0 ** (-(np.arange(len(sizes)) % 5))
        gpu = SegGpu(seg_off, seg_k, caps, inplace)
        eps = np.zeros(int(seg_off[-1]), np.float32)
        for step in range(3):
            g = seg_grad(seg_off, 300 + n, step, sig)
            gpu.set_residual(eps)
            eps = check_segmented(mode, gpu, g, eps, what=f"layout {n} mode {mode} step {step}")


@pytest.mark.parametrize("mode", [0, 1])
def test_ties_and_output_ranges_too_small(mode):
    sizes = [500, 3000, 64, 9000]
    seg_off, seg_k, caps = layout(sizes, rho_den=10)
    caps[1] = 5        # Top_k: cap < k -> nothing; Gaussian_k: count > cap -> nothing
    caps[2] = 0
    rng = np.random.default_rng(4)
    g = rng.integers(-3, 4, int(seg_off[-1])).astype(np.float32)   # heavy ties in every segment
    gpu = SegGpu(seg_off, seg_k, caps)
    eps = np.zeros_like(g)
    check_segmented(mode, gpu, g, eps, what=f"ties mode {mode}")
    res = S.decode_results(gpu.b.result)
    if mode == 0:
        assert res[1]["flags"] & S.F_OVERFLOW and res[1]["nnz"] == 0
    # Gaussian data: the count (about k = 300) cannot fit a range of 5
    g = synth.normal(int(seg_off[-1]), 6, 0, 1.0)
    gpu.set_residual(eps)
    check_segmented(mode, gpu, g, eps, what=f"overflow mode {mode}")
    res = S.decode_results(gpu.b.result)
    assert res[1]["flags"] & S.F_OVERFLOW and res[1]["nnz"] == 0
    assert res[2]["flags"] & S.F_OVERFLOW and res[2]["nnz"] == 0
    assert res[0]["nnz"] > 0 and res[3]["nnz"] > 0


@pytest.mark.parametrize("inplace", [False, True])
def test_topk_ranked_ties_in_segments_of_many_tiles(inplace):
    """Segments of 74, 171 and 65 tiles (several groups of 64 tiles each) filled with a handful
    of values: the k-th key of a segment is shared by thousands of entries spread over all its
    tiles, and only the lowest-index ones are kept."""
    sizes = [300_000, 5, 700_001, 4096 * 64 + 1, 17]
    rng = np.random.default_rng(8)
    d = int(np.sum(sizes))
    vecs = [rng.integers(-3, 4, d).astype(np.float32), np.full(d, 0.5, np.float32)]
    late = np.zeros(d, np.float32)
    late[300_005 + 690_000:300_005 + 700_001] = -1.0   # every tie of segment 2 in its last tiles
    vecs.append(late)
    for rho_den in (3, 1000):
        seg_off, seg_k, caps = layout(sizes, rho_den=rho_den, cap_mult=1)
        gpu = SegGpu(seg_off, seg_k, caps, inplace)
        for n, g in enumerate(vecs):
            eps = np.zeros(d, np.float32)
            gpu.set_residual(eps)
            check_segmented(0, gpu, g, eps, what=f"ties vec {n} rho 1/{rho_den} inplace={inplace}")


@pytest.mark.parametrize("mode", [0, 1])
def test_twenty_thousand_tiny_segments(mode):
    """Many more segments than tiles of any one of them: sizes 1..120, k_l from 1 to the whole
    segment, a few output ranges too small."""
    rng = np.random.default_rng(31 + mode)
    L = 20_000
    sizes = rng.integers(1, 121, L).astype(np.int64)
    seg_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    seg_k = np.minimum(sizes, np.maximum(1, (sizes * rng.uniform(0, 1, L)).astype(np.int64)))
    caps = np.where(rng.random(L) < 0.05, 0, 2 * sizes + 2).astype(np.int64)
    d = int(seg_off[-1])
    g = (rng.standard_normal(d) * 10.0 ** rng.integers(-4, 2, d)).astype(np.float32)
    g[rng.integers(0, d, d // 20)] = 0.5     # ties
    eps = np.zeros(d, np.float32)
    gpu = SegGpu(seg_off, seg_k, caps)
    for step in range(2):
        gpu.set_residual(eps)
        eps = check_segmented(mode, gpu, g, eps, what=f"20000 segments mode {mode} step {step}")


def test_invalid_segments_are_flagged_and_produce_nothing():
    d = 10_000
    seg_off = np.array([0, 3000, 2000, 10_000], np.int64)   # segment 1 runs backwards
    seg_k = np.array([30, 10, 9000], np.int64)              # segment 2: k > length
    caps = np.array([200, 200, 200], np.int64)
    gpu = SegGpu(seg_off, seg_k, caps)
    g = synth.normal(d, 5, 0, 1.0)
    gpu.b.residual.zero_()
    for mode in (0, 1):
        out = gpu.step(mode, g)
        assert out["res"][0]["flags"] == 0 and out["res"][0]["nnz"] > 0
        for l in (1, 2):
            assert out["res"][l]["flags"] == S.F_BADSEGMENT and out["res"][l]["nnz"] == 0
        assert np.all(out["idx"][200:] == -1)
        gpu.b.residual.zero_()


def test_segments_that_step_back_behind_an_earlier_offset_are_flagged():
    """A layout whose offsets are not monotone: a segment that is valid on its own but starts
    before an earlier offset could overlap an earlier segment, so it is flagged and skipped; the
    segments before the step back are processed as usual."""
    d = 20_000
    #                     seg0 [0,9000)  seg1 backwards  seg2 [5000,6000)  seg3 [6000,20000)
    seg_off = np.array([0, 9000, 5000, 6000, 20_000], np.int64)
    seg_k = np.array([9, 1, 1, 14], np.int64)
    caps = np.array([100, 100, 100, 100], np.int64)
    gpu = SegGpu(seg_off, seg_k, caps)
    g = synth.normal(d, 6, 0, 1.0)
    for mode in (0, 1):
        gpu.b.residual.zero_()
        gpu.b.acc.fill_(float("nan"))
        out = gpu.step(mode, g)
        assert out["res"][0]["flags"] == 0 and out["res"][0]["nnz"] > 0
        for l in (1, 2, 3):
            assert out["res"][l]["flags"] == S.F_BADSEGMENT and out["res"][l]["nnz"] == 0, l
        assert np.all(out["idx"][100:] == -1)
        # segment 0 alone was processed: its stretch equals the flat oracle on it, the rest of
        # acc was never written
        acc_o = O.accumulate(g[:9000], np.zeros(9000, np.float32))
        assert same_bits(out["acc"][:9000], acc_o)
        assert np.all(np.isnan(out["acc"][9000:]))
        if mode == 0:
            idx_o, val_o, eps_o, _ = O.topk(acc_o, 9)
        else:
            idx_o, val_o, eps_o, ro = O.gaussiank(acc_o, 9, cap=100)
        n = int(out["res"][0]["nnz"])
        assert np.array_equal(np.sort(out["idx"][:n].view(np.uint32)), idx_o)
        assert same_bits(out["eps"][:9000], eps_o)
        assert not out["eps"][9000:].any()


@pytest.mark.parametrize("mode", [0, 1])
def test_cfg4_segmented_workload(mode):
    """54 segments summing to d = 25,557,032, per-segment scales over three decades, all
    segments in one launch, 20 error-feedback iterations."""
    wl = synth.workload("cfg4_segmented")
    caps = np.maximum(4 * wl.seg_k, 1024)
    gpu = SegGpu(wl.seg_off, wl.seg_k, caps)
    eps = np.zeros(wl.d, np.float32)
    g = np.empty(wl.d, np.float32)
    for step in range(wl.steps):
        wl.grad(step, out=g)
        eps = check_segmented(mode, gpu, g, eps, what=f"cfg4 mode {mode} step {step}")
        progress(f"cfg4 mode {mode} step {step} ok")


def test_layer_wise_calls_take_the_short_launch_sequences():
    """The kernels behind a call are visible through the trace: three launches for
    Gaussian_k (up to 256 segments: the accumulate kernel has the setup in it), seven launches for Top_k with a separate accumulator (candidate filtering; the
    setup kernel also clears the histograms), the long general sequence only in place."""
    seg_off, seg_k, caps = layout([100_000, 7, 250_001, 64])
    want = {(1, False): ["accum_moments", "gk_count", "gk_compact"],
            (0, False): ["seg_setup", "topk_accum_hist", "topk_filter", "topk_cand2",
                         "topk_cand3", "topk_final", "topk_compact"]}
    g = seg_grad(seg_off, 5, 0, [1e-2, 1.0, 1e-3, 1e-1])
    for inplace in (False, True):
        gpu = SegGpu(seg_off, seg_k, caps, inplace)
        for mode in (1, 0):
            tr = S.Trace()
            gpu.set_residual(np.zeros_like(g))
            gpu.step(mode, g, trace=tr)
            names = [n for n, _ in tr.stages()]
            if (mode, inplace) in want:
                assert names == want[(mode, inplace)], names
            elif mode == 1:
                assert names == want[(1, False)], names
            else:
                assert len(names) == 12 and names[-1] == "topk_compact", names

"""GPU parity of the layer-wise Gaussian_k call where the count kernel also lists each tile's
entries above its segment's thres0 and writes the residual (vectors of 6 M elements and more, up
to 1024 segments): a segment whose walk ended at thres0 or above takes its pairs from the lists,
the others (and a segment one of whose stretches of the list buffer ran out) are compacted by
streaming acc.  Results must not depend on the way, so every case is compared with the CPU oracle
bit for bit, and the way each segment took (two informational flag bits) is checked against what
the input was built to provoke."""
import numpy as np
import pytest
import torch

from gpu_harness import SegGpu, check_segmented
from paper_1911_08772_amd import sparsify as S
from paper_1911_08772_amd import synth

pytestmark = pytest.mark.gpu


def ways(gpu):
    return [int(r["flags"]) & S.F_WAY for r in S.decode_results(gpu.b.result)]


def layout(sizes, rho=0.001):
    sizes = np.asarray(sizes, np.int64)
    seg_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    seg_k = np.maximum(1, np.ceil(sizes * rho)).astype(np.int64)
    caps = np.maximum(4 * seg_k, 64)
    return seg_off, seg_k, caps


@pytest.mark.parametrize("inplace", [False, True])
def test_resnet50_sized_layout_takes_the_lists(inplace):
    wl = synth.workload("cfg4_segmented")
    caps = np.maximum(4 * wl.seg_k, 1024)
    gpu = SegGpu(wl.seg_off, wl.seg_k, caps, inplace=inplace)
    sizes = np.diff(wl.seg_off)
    eps = np.zeros(wl.d, np.float32)
    for step in range(4):
        gpu.set_residual(eps)
        eps = check_segmented(1, gpu, wl.grad(step), eps, what=f"cfg4 inplace={inplace} step {step}")
        w = ways(gpu)
        assert all(x in (S.F_SHORTLIST, S.F_SHORTLIST_MISS) for x in w), w
        # fresh bell-shaped segments of some length are in the band at thres0
        if step == 0:
            assert all(x == S.F_SHORTLIST for x, n in zip(w, sizes) if n >= 100_000), (w, sizes)
        assert sum(x == S.F_SHORTLIST for x in w) >= len(w) // 2, w


def test_segments_decide_for_themselves():
    """A uniform segment (its walk ends far below thres0), a segment around -5 (thres0 negative),
    an all-zero one and a one-element one between bell-shaped ones: those four stream, the others
    take their lists; ragged offsets."""
    sizes = [2_000_003, 700_001, 1_500_000, 1, 4097, 900_000, 1_100_007, 333]
    seg_off, seg_k, caps = layout(sizes)
    caps[1] = sizes[1]  # the uniform segment ends with a third of its entries selected
    caps[5] = sizes[5]  # every entry of the segment around -5 exceeds a negative threshold
    d = int(seg_off[-1])
    rng = np.random.default_rng(3)
    g = synth.normal(d, 71, 0, 0.01)
    g[seg_off[1]:seg_off[2]] = rng.uniform(-1, 1, sizes[1]).astype(np.float32)
    g[seg_off[4]:seg_off[5]] = 0.0
    g[seg_off[5]:seg_off[6]] = (rng.standard_normal(sizes[5]) * 0.01 - 5.0).astype(np.float32)
    gpu = SegGpu(seg_off, seg_k, caps)
    zero = np.zeros(d, np.float32)
    gpu.set_residual(zero)
    check_segmented(1, gpu, g, zero, what="mixed segments")
    w = ways(gpu)
    assert w[0] == w[2] == w[6] == S.F_SHORTLIST, w
    assert w[1] == w[4] == w[5] == S.F_SHORTLIST_MISS, w
    assert w[3] in (S.F_SHORTLIST, S.F_SHORTLIST_MISS) and w[7] in (S.F_SHORTLIST, S.F_SHORTLIST_MISS), w


def test_a_stretch_that_runs_out_leaves_its_own_segment_streaming():
    sizes = [3_000_000, 2_000_000, 1_500_000]
    seg_off, seg_k, caps = layout(sizes)
    d = int(seg_off[-1])
    rng = np.random.default_rng(4)
    g = rng.standard_normal(d).astype(np.float32)
    g[3_100_000:3_300_000] *= np.float32(100.0)   # half of this stretch exceeds its segment's thres0
    caps[1] = sizes[1]
    gpu = SegGpu(seg_off, seg_k, caps)
    zero = np.zeros(d, np.float32)
    gpu.set_residual(zero)
    check_segmented(1, gpu, g, zero, what="one loud stretch")
    assert ways(gpu) == [S.F_SHORTLIST, S.F_SHORTLIST_MISS, S.F_SHORTLIST]


def test_the_lists_can_be_declined():
    sizes = [3_000_000, 2_000_001, 1_499_999]
    seg_off, seg_k, caps = layout(sizes)
    d = int(seg_off[-1])
    g = synth.normal(d, 72, 0, 0.01)
    eps = synth.normal(d, 73, 0, 0.003)
    gpu = SegGpu(seg_off, seg_k, caps)
    for mode, kw in ((1, {"short_list": -1}), (1, {"error_norms": True})):
        gpu.set_residual(eps)
        check_segmented(mode, gpu, g, eps, what=f"mode {mode} {kw}", **kw)
        assert ways(gpu) == [0, 0, 0], (mode, kw)
    for kw in ({"tile_chunks": 1}, {"tile_chunks": 2}, {"tail_div": 1.0}):
        gpu.set_residual(eps)
        check_segmented(1, gpu, g, eps, what=f"{kw}", **kw)
        assert ways(gpu) == [S.F_SHORTLIST] * 3, kw
    # a forced tile length whose ragged tiles the run table does not hold
    gpu.set_residual(eps)
    check_segmented(1, gpu, g, eps, what="tile_chunks=64", tile_chunks=64)
    assert ways(gpu) == [0, 0, 0]
    small = S.workspace_bytes_min(d, 3)
    assert small < gpu.b.workspace_nbytes
    gpu.b.workspace = torch.empty(small, dtype=torch.uint8, device="cuda:0")
    gpu.set_residual(eps)
    check_segmented(1, gpu, g, eps, what="small workspace")
    assert ways(gpu) == [0, 0, 0]


def test_more_segments_than_the_run_table_is_sized_for():
    L = 1025
    sizes = np.full(L, 6000, np.int64)
    sizes[0] = 6_200_000 - int(sizes[1:].sum())
    seg_off, seg_k, caps = layout(sizes)
    d = int(seg_off[-1])
    assert S.workspace_bytes(d, L) == S.workspace_bytes_min(d, L)
    g = synth.normal(d, 74, 0, 0.01)
    zero = np.zeros(d, np.float32)
    gpu = SegGpu(seg_off, seg_k, caps)
    gpu.set_residual(zero)
    check_segmented(1, gpu, g, zero, what="1025 segments")
    assert set(ways(gpu)) == {0}


def test_a_layer_wise_call_with_lists_can_be_captured_in_a_hip_graph():
    """Every segment's way is decided on the device, so a captured call replays with or without
    the lists as each replay's data asks."""
    from gpu_harness import same_bits
    from oracle import oracle as O
    sizes = [3_000_000, 2_000_001, 1_499_999]
    seg_off, seg_k, caps = layout(sizes)
    d, L = int(seg_off[-1]), 3
    out_off = np.concatenate([[0], np.cumsum(caps)]).astype(np.int64)
    ocap = int(out_off[-1])
    b = S.Buffers.allocate(d, ocap, L)
    grad = torch.zeros(d, device="cuda:0")
    d_off, d_k, d_oo = (torch.from_numpy(x).to("cuda:0") for x in (seg_off, seg_k, out_off))

    def call():
        S.sparsify_segmented(L, d, d_off, d_k, 1, grad, b.residual, b.acc, b.out_idx, b.out_val, d_oo,
                             ocap, b.result, b.workspace, b.workspace_nbytes)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):   # warm-up outside capture (first-call queries of the runtime)
        call()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    b.residual.zero_()
    eps = np.zeros(d, np.float32)
    rng = np.random.default_rng(8)
    for step in range(4):
        g = synth.normal(d, 83, step, 0.01)
        if step == 2:   # the middle segment uniform: its walk ends below thres0, it alone streams
            g[seg_off[1]:seg_off[2]] = rng.uniform(-1, 1, sizes[1]).astype(np.float32)
            eps = np.zeros(d, np.float32)
            b.residual.zero_()
        grad.copy_(torch.from_numpy(g))
        b.out_idx.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        acc_o = O.accumulate(g, eps)
        idx_o, val_o, eps, res_o = O.segmented(acc_o, seg_off, seg_k, 1, out_off)
        res = S.decode_results(b.result)
        got_idx, got_val = b.out_idx.cpu().numpy(), b.out_val.cpu().numpy()
        for l in range(L):
            n, o0 = res_o[l].nnz, int(out_off[l])
            assert int(res[l]["nnz"]) == n and int(res[l]["rounds"]) == res_o[l].rounds, (step, l)
            assert np.array_equal(got_idx[o0:o0 + n].view(np.uint32), idx_o[o0:o0 + n]), (step, l)
            assert same_bits(got_val[o0:o0 + n], val_o[o0:o0 + n]), (step, l)
        w = [int(r["flags"]) & S.F_WAY for r in res]
        if step == 2:
            assert w == [S.F_SHORTLIST, S.F_SHORTLIST_MISS, S.F_SHORTLIST], w
        else:
            assert all(x in (S.F_SHORTLIST, S.F_SHORTLIST_MISS) for x in w) and S.F_SHORTLIST in w, w
        assert same_bits(b.residual.cpu().numpy(), eps), step
        assert same_bits(b.acc.cpu().numpy(), acc_o), step
        _ = (b.acc * 2).sum().item()   # unrelated eager work between replays

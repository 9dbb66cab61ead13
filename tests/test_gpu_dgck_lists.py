"""GPU parity of DGC_k (Sec. 3.3 / Sec. 4.3) where the library draws the sample first and lets the
accumulate pass list the entries that reach the sample's threshold (vectors of 6 M elements and
more, k up to d/80, strides from 10): results must not depend on whether those lists end up
being used, so every case is compared with the CPU oracle bit for bit, and the way the call took
(two informational flag bits) is checked against what the input was built to provoke."""
import numpy as np
import pytest
import torch

from gpu_harness import FlatGpu, check_flat, same_bits
from oracle import oracle as O
from paper_1911_08772_amd import sparsify as S
from paper_1911_08772_amd import synth

pytestmark = pytest.mark.gpu


def way(gpu):
    return int(S.decode_results(gpu.b.result)[0]["flags"]) & S.F_WAY


def rounds(gpu):
    return int(S.decode_results(gpu.b.result)[0]["rounds"])


@pytest.mark.parametrize("d", [6_000_000, 8_388_608 + 1, 6_000_000 + 4095])
def test_typical_vectors_take_the_lists(d):
    gpu = FlatGpu(d, cap=d // 80 + 16)
    eps = np.zeros(d, np.float32)
    seen = set()
    step = 0
    for k in (d // 1000, d // 100, 1):  # a short error-feedback chain
        for stride in (100, 1000, 10):
            g = synth.normal(d, 950 + step, d, 0.01)
            gpu.set_residual(eps)
            eps = check_flat("dgck", gpu, g, eps, k, what=f"d={d} k={k} S={stride}",
                             sample_stride=stride, sample_seed=step)
            assert way(gpu) == S.F_SHORTLIST, (d, k, stride)
            seen.add(rounds(gpu))
            step += 1
    assert seen == {1, 2}   # with and without the second selection


def test_heavy_tails_and_ranked_ties_from_the_lists():
    d, k = 7_000_003, 7000
    gpu = FlatGpu(d, cap=2 * k)
    zero = np.zeros(d, np.float32)
    x = synth.student_t3(d, 57, 0, 1e-3)
    check_flat("dgck", gpu, x, zero, k, what="student-t", sample_seed=3)
    assert way(gpu) == S.F_SHORTLIST
    # 9000 entries share one magnitude (both signs, spread over the vector, in runs and alone)
    # and the sample's threshold falls on it: all of them are kept, which is more than k, and
    # the second selection keeps the lowest-index ones
    rng = np.random.default_rng(12)
    y = synth.normal(d, 58, 0, 0.01)
    where = np.unique(np.concatenate([rng.integers(0, d, 7000), np.arange(2_345_000, 2_347_000)]))
    y[where] = np.float32(0.0625)
    y[where[::3]] = np.float32(-0.0625)
    y[rng.integers(0, d, 300)] = np.float32(0.5)      # a few entries above the ties
    gpu.set_residual(zero)
    check_flat("dgck", gpu, y, zero, k, what="ranked ties", sample_seed=4)
    res = S.decode_results(gpu.b.result)[0]
    assert int(res["topk_key"]) == int(np.float32(0.0625).view(np.uint32)) and way(gpu) == S.F_SHORTLIST
    assert rounds(gpu) == 2 and 0 < int(res["topk_ties_taken"]) < where.size


def test_vectors_whose_kept_entries_no_list_holds():
    d, k, stride, seed = 6_300_000 + 77, 6300, 100, 9
    rng = np.random.default_rng(78)
    zero = np.zeros(d, np.float32)
    gpu = FlatGpu(d, cap=d)  # (DGC_k keeps every entry that reaches the threshold: up to d pairs)
    vecs = {"zeros": (np.zeros(d, np.float32), S.F_SHORTLIST_MISS),
            "constant": (np.full(d, 0.375, np.float32), S.F_SHORTLIST_MISS),
            "small_ints": (rng.integers(-3, 4, d).astype(np.float32), S.F_SHORTLIST_MISS)}
    # zero wherever the sample looks, large elsewhere: the threshold is 0 and everything is kept
    v = rng.standard_normal(d).astype(np.float32)
    pos = O.dgck(v, k, stride, seed, want_positions=True)[4]
    v[pos] = 0.0
    vecs["sample_sees_zeros"] = (v, S.F_SHORTLIST_MISS)
    n = rng.standard_normal(d).astype(np.float32)
    n[rng.integers(0, d, 3)] = np.float32(np.nan)
    vecs["nans"] = (n, S.F_SHORTLIST)
    # one stretch a hundred times larger than the rest: every kept entry sits there, and the few
    # waves that stream it may or may not have room for their lists
    w = rng.standard_normal(d).astype(np.float32)
    w[1_000_000:1_200_000] *= np.float32(100.0)
    vecs["one_loud_stretch"] = (w, None)
    for name, (acc, expected) in vecs.items():
        gpu.set_residual(zero)
        check_flat("dgck", gpu, acc, zero, k, what=name, sample_stride=stride, sample_seed=seed)
        assert way(gpu) in (S.F_SHORTLIST, S.F_SHORTLIST_MISS), name
        if expected is not None:
            assert way(gpu) == expected, name


def test_the_lists_can_be_declined():
    """short_list = -1, the error norms, k beyond d/80, a sample too long for the list buffer
    and a workspace of the smaller size all take the eleven-launch form: same results, no way
    reported."""
    d, k = 6_100_000, 6100
    g = synth.normal(d, 43, 0, 0.01)
    eps = synth.normal(d, 44, 0, 0.003)
    gpu = FlatGpu(d, cap=d // 20)
    for kk, kw in ((k, {"short_list": -1}), (k, {"error_norms": True}), (d // 79, {}),
                   (k, {"sample_stride": 3})):
        gpu.set_residual(eps)
        check_flat("dgck", gpu, g, eps, kk, what=f"{kw} k={kk}", **kw)
        assert way(gpu) == 0, (kk, kw)
    for tc in (2, 5):
        gpu.set_residual(eps)
        check_flat("dgck", gpu, g, eps, k, what=f"tile_chunks={tc}", tile_chunks=tc)
        assert way(gpu) == S.F_SHORTLIST, tc
    small = S.workspace_bytes_min(d, 1)
    assert small < gpu.b.workspace_nbytes
    gpu.b.workspace = torch.empty(small, dtype=torch.uint8, device="cuda:0")
    gpu.set_residual(eps)
    check_flat("dgck", gpu, g, eps, k, what="small workspace")
    assert way(gpu) == 0


def test_a_call_with_lists_can_be_captured_in_a_hip_graph():
    """The way a call takes is decided on the device, so a captured call replays with or without
    the lists as each replay's data asks: typical gradients take them, an all-zero one does not."""
    d, k = 6_100_000, 6100
    b = S.Buffers.allocate(d, d)
    grad = torch.zeros(d, device="cuda:0")

    def call():
        S.sparsify_dgck(d, k, grad, b.residual, b.acc, b.out_idx, b.out_val, d, b.result, b.workspace,
                        b.workspace_nbytes, sample_seed=21)
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
    for step in range(5):
        g = np.zeros(d, np.float32) if step == 2 else synth.normal(d, 79, step, 0.01)
        if step == 2:
            eps = np.zeros(d, np.float32)   # with a zero residual acc is all zero: everything is kept
            b.residual.zero_()
        grad.copy_(torch.from_numpy(g))
        b.out_idx.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        acc_o = O.accumulate(g, eps)
        idx_o, val_o, eps, ro = O.dgck(acc_o, k, 100, 21)
        res = S.decode_results(b.result)[0]
        assert int(res["nnz"]) == ro.nnz and int(res["rounds"]) == ro.rounds, step
        assert (int(res["flags"]) & S.F_WAY) == (S.F_SHORTLIST_MISS if step == 2 else S.F_SHORTLIST), step
        assert np.array_equal(b.out_idx[:ro.nnz].cpu().numpy().view(np.uint32), idx_o), step
        assert same_bits(b.out_val[:ro.nnz].cpu().numpy(), val_o), step
        assert same_bits(b.residual.cpu().numpy(), eps), step
        assert same_bits(b.acc.cpu().numpy(), acc_o), step
        _ = (b.acc * 2).sum().item()   # unrelated eager work between replays

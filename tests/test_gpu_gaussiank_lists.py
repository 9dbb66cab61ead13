"""GPU parity of flat Gaussian_k (Algorithm 1) where the count kernel also lists the entries above
thres0 and writes the residual, so that the compact kernel can write the pairs from the lists
(vectors of 6 M elements and more, k up to d/20).  Whether a call ends up using its lists depends
on the data (a walk that ends below thres0, a thres0 that is not positive and a list that runs
out of room all leave them unused); the results must not, so every case is compared with the CPU
oracle bit for bit, and the way the call took (two informational flag bits) is checked against
what the input was built to provoke."""
import numpy as np
import pytest
import torch

from gpu_harness import FlatGpu, check_flat, same_bits
from oracle import oracle as O
from paper_1911_08772_amd import sparsify as S
from paper_1911_08772_amd import synth

pytestmark = pytest.mark.gpu


def rec(gpu):
    return S.decode_results(gpu.b.result)[0]


def way(gpu):
    return int(rec(gpu)["flags"]) & S.F_WAY


@pytest.mark.parametrize("inplace", [False, True])
@pytest.mark.parametrize("d", [6_000_000, 8_388_608 + 1, 6_000_000 + 4095])
def test_error_feedback_chains_take_the_lists(d, inplace):
    k = d // 1000
    gpu = FlatGpu(d, cap=4 * k, inplace=inplace)
    eps = np.zeros(d, np.float32)
    finals = set()
    for step in range(6):
        g = synth.normal(d, 970 + step, d, 0.01)
        gpu.set_residual(eps)
        eps = check_flat("gaussiank", gpu, g, eps, k, what=f"d={d} inplace={inplace} step {step}")
        assert way(gpu) == S.F_SHORTLIST, (d, inplace, step)
        r = rec(gpu)
        finals.add(round(float(r["thres_f32"]) / float(r["thres0"]), 3))
    assert finals == {1.0, 1.125}, finals  # one evaluation on a fresh vector; four under error feedback


def two_levels(d, k, upper, lower, rng):
    """`upper` entries of magnitude 1 and `lower` of magnitude 0.05 in small noise: thres0 falls
    between the two levels (0.074 for upper = k/2), so the walk's outcome is a matter of counts."""
    v = (rng.standard_normal(d) * 1e-6).astype(np.float32)
    where = rng.choice(d, upper + lower, replace=False)
    v[where[:upper]] = np.float32(1.0)
    v[where[upper:]] = np.float32(0.05)
    v[where[::2]] *= np.float32(-1.0)
    return v


@pytest.mark.parametrize("inplace", [False, True])
def test_walks_that_end_below_thres0_leave_the_lists_unused(inplace):
    d, k = 6_200_000 + 13, 6200
    rng = np.random.default_rng(5)
    zero = np.zeros(d, np.float32)
    gpu = FlatGpu(d, cap=4 * k, inplace=inplace)
    # k/2 above thres0, then 1.2 k above half of it: in the band at the second evaluation
    check_flat("gaussiank", gpu, two_levels(d, k, k // 2, 7 * k // 10, rng), zero, k, what="ends at 0.5 thres0")
    r = rec(gpu)
    assert int(r["rounds"]) == 2 and float(r["thres_f32"]) < float(r["thres0"]) and way(gpu) == S.F_SHORTLIST_MISS
    # k/2 and then 1.5 k: too few, too many, too few, too many: ends at 0.375 thres0
    gpu.set_residual(zero)
    check_flat("gaussiank", gpu, two_levels(d, k, k // 2, k, rng), zero, k, what="ends at 0.375 thres0")
    r = rec(gpu)
    assert int(r["rounds"]) == 4 and float(r["thres_f32"]) < float(r["thres0"]) and way(gpu) == S.F_SHORTLIST_MISS
    # 0.7 k above thres0: in the band at once, the lists serve
    gpu.set_residual(zero)
    check_flat("gaussiank", gpu, two_levels(d, k, 7 * k // 10, k, rng), zero, k, what="ends at thres0")
    assert int(rec(gpu)["rounds"]) == 1 and way(gpu) == S.F_SHORTLIST


def test_vectors_that_no_list_serves():
    d, k = 6_300_000 + 77, 6300
    rng = np.random.default_rng(79)
    zero = np.zeros(d, np.float32)
    gpu = FlatGpu(d, cap=d)
    vecs = {}
    vecs["zeros"] = (np.zeros(d, np.float32), S.F_SHORTLIST_MISS)            # thres0 = 0
    # mean -5, small spread: thres0 is negative, every entry exceeds every threshold
    vecs["negative_thres0"] = ((rng.standard_normal(d) * 0.01 - 5.0).astype(np.float32), S.F_SHORTLIST_MISS)
    # uniform: no tail at all, the walk ends far below thres0 with a quarter of the vector selected
    vecs["uniform"] = (rng.uniform(-1, 1, d).astype(np.float32), S.F_SHORTLIST_MISS)
    n = rng.standard_normal(d).astype(np.float32)
    n[rng.integers(0, d, 3)] = np.float32(np.nan)                            # moments are NaN
    vecs["nans"] = (n, S.F_SHORTLIST_MISS)
    # one stretch a hundred times larger than the rest: half of it exceeds thres0, and the waves
    # that stream it run out of room for their lists
    w = rng.standard_normal(d).astype(np.float32)
    w[1_000_000:1_200_000] *= np.float32(100.0)
    vecs["one_loud_stretch"] = (w, S.F_SHORTLIST_MISS)
    vecs["student_t"] = (synth.student_t3(d, 59, 0, 1e-3), S.F_SHORTLIST)
    for name, (acc, expected) in vecs.items():
        gpu.set_residual(zero)
        check_flat("gaussiank", gpu, acc, zero, k, what=name)
        assert way(gpu) == expected, name


def test_more_survivors_than_cap_with_lists():
    """More survivors than `cap`: nothing is selected and the residual is acc, whichever way."""
    d, k = 6_100_000, 6100
    g = synth.normal(d, 45, 0, 0.01)
    zero = np.zeros(d, np.float32)
    gpu = FlatGpu(d, cap=100)
    check_flat("gaussiank", gpu, g, zero, k, what="cap 100")
    r = rec(gpu)
    assert int(r["flags"]) & S.F_OVERFLOW and int(r["nnz"]) == 0 and way(gpu) == S.F_SHORTLIST


def test_the_lists_can_be_declined():
    d, k = 6_100_000, 6100
    g = synth.normal(d, 46, 0, 0.01)
    eps = synth.normal(d, 47, 0, 0.003)
    gpu = FlatGpu(d, cap=d // 20)
    for kk, kw in ((k, {"short_list": -1}), (k, {"error_norms": True}), (d // 19, {})):
        gpu.set_residual(eps)
        check_flat("gaussiank", gpu, g, eps, kk, what=f"{kw} k={kk}", **kw)
        assert way(gpu) == 0, (kk, kw)
    gpu.set_residual(eps)
    check_flat("gaussiank", gpu, g, eps, d // 21, what="k = d/21")   # up to a twentieth of the vector
    assert way(gpu) in (S.F_SHORTLIST, S.F_SHORTLIST_MISS)
    for kw in ({"tile_chunks": 1}, {"tile_chunks": 2}, {"tile_chunks": 5}, {"tail_div": 1.0}, {"ddof": 0}):
        gpu.set_residual(eps)
        check_flat("gaussiank", gpu, g, eps, k, what=f"{kw}", **kw)
        assert way(gpu) == S.F_SHORTLIST, kw
    small = S.workspace_bytes_min(d, 1)
    assert small < gpu.b.workspace_nbytes
    gpu.b.workspace = torch.empty(small, dtype=torch.uint8, device="cuda:0")
    gpu.set_residual(eps)
    check_flat("gaussiank", gpu, g, eps, k, what="small workspace")
    assert way(gpu) == 0


def test_a_call_with_lists_can_be_captured_in_a_hip_graph():
    """The way a call takes is decided on the device, so a captured call replays with or without
    the lists as each replay's data asks: typical gradients take them, an all-zero one does not."""
    d, k = 6_100_000, 6100
    cap = 4 * k
    b = S.Buffers.allocate(d, cap)
    grad = torch.zeros(d, device="cuda:0")

    def call():
        S.sparsify_gaussiank(d, k, grad, b.residual, b.acc, b.out_idx, b.out_val, cap, b.result,
                             b.workspace, b.workspace_nbytes)
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
        g = np.zeros(d, np.float32) if step == 2 else synth.normal(d, 81, step, 0.01)
        if step == 2:
            eps = np.zeros(d, np.float32)   # with a zero residual acc is all zero: thres0 = 0
            b.residual.zero_()
        grad.copy_(torch.from_numpy(g))
        b.out_idx.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        acc_o = O.accumulate(g, eps)
        idx_o, val_o, eps, ro = O.gaussiank(acc_o, k, cap=cap)
        res = S.decode_results(b.result)[0]
        assert int(res["nnz"]) == ro.nnz and int(res["rounds"]) == ro.rounds, step
        assert (int(res["flags"]) & S.F_WAY) == (S.F_SHORTLIST_MISS if step == 2 else S.F_SHORTLIST), step
        assert np.array_equal(b.out_idx[:ro.nnz].cpu().numpy().view(np.uint32), idx_o), step
        assert same_bits(b.out_val[:ro.nnz].cpu().numpy(), val_o), step
        assert same_bits(b.residual.cpu().numpy(), eps), step
        assert same_bits(b.acc.cpu().numpy(), acc_o), step
        _ = (b.acc * 2).sum().item()   # unrelated eager work between replays

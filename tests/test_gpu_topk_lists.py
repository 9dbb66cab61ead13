"""GPU parity of flat Top_k where the library builds short lists in the accumulate pass (vectors
of 6 M elements and more, k up to d/80): the results must not depend on whether the lists end
up being used, so every case is compared with the CPU oracle bit for bit, and the way the call
took (reported in two informational flag bits) is checked against what the input was built to
provoke: typical vectors take the lists; vectors that defeat the guess the lists are built on
(fewer than k entries above the listing key, a list that runs out of room) end in the passes over
acc."""
import numpy as np
import pytest
import torch

from gpu_harness import FlatGpu, check_flat
from paper_1911_08772_amd import sparsify as S
from paper_1911_08772_amd import synth

pytestmark = pytest.mark.gpu

D0 = 6_000_000  # the shortest vector that gets lists


def way(gpu):
    return int(S.decode_results(gpu.b.result)[0]["flags"]) & S.F_WAY


@pytest.mark.parametrize("inplace", [False, True])
@pytest.mark.parametrize("d", [D0, 8_388_608, 8_388_608 + 1, 6_000_000 + 4095, 9_000_017])
def test_typical_vectors_take_the_lists(d, inplace):
    gpu = FlatGpu(d, cap=d // 100 + 16, inplace=inplace)
    eps = np.zeros(d, np.float32)
    for step, k in enumerate((d // 1000, d // 100, 1)):  # a short error-feedback chain
        g = synth.normal(d, 900 + step, d, 0.01)
        gpu.set_residual(eps)
        eps = check_flat("topk", gpu, g, eps, k, what=f"d={d} inplace={inplace} k={k}")
        assert way(gpu) == S.F_SHORTLIST, (d, inplace, k)


@pytest.mark.parametrize("inplace", [False, True])
def test_heavy_tails_and_ranked_ties_from_the_lists(inplace):
    d, k = 7_000_003, 7000
    gpu = FlatGpu(d, cap=k, inplace=inplace)
    zero = np.zeros(d, np.float32)
    x = synth.student_t3(d, 55, 0, 1e-3)
    check_flat("topk", gpu, x, zero, k, what="student-t")
    assert way(gpu) == S.F_SHORTLIST
    # 8000 entries share the k-th magnitude (both signs, spread over the whole vector, in runs and
    # alone): only the lowest-index ones are kept, and those come from the lists in index order
    rng = np.random.default_rng(11)
    y = synth.normal(d, 56, 0, 0.01)
    where = np.unique(np.concatenate([rng.integers(0, d, 8000), np.arange(1_234_000, 1_237_000)]))
    y[where] = np.float32(0.0625)
    y[where[::3]] = np.float32(-0.0625)
    y[rng.integers(0, d, 300)] = np.float32(0.5)      # a few entries above the ties
    gpu.set_residual(zero)
    check_flat("topk", gpu, y, zero, k, what="ranked ties")
    res = S.decode_results(gpu.b.result)[0]
    assert int(res["topk_key"]) == int(np.float32(0.0625).view(np.uint32)) and way(gpu) == S.F_SHORTLIST
    assert 0 < int(res["topk_ties_taken"]) < where.size


def defeating_vectors(d, rng):
    out = {}
    out["zeros"] = np.zeros(d, np.float32)
    out["constant"] = np.full(d, 0.375, np.float32)
    # small integers: the k-th magnitude is also the largest, nothing lies above the listing key
    out["small_ints"] = rng.integers(-3, 4, d).astype(np.float32)
    # zero wherever the sample looks (four consecutive entries every d/1024 elements), large
    # elsewhere: the listing key is 0 and the lists would have to hold the whole vector
    v = rng.standard_normal(d).astype(np.float32)
    stride = (d // 4) // 1024 * 4
    for s in range(1024):
        v[s * stride: s * stride + 4] = 0.0
    out["sample_sees_zeros"] = v
    n = rng.standard_normal(d).astype(np.float32)
    n[rng.integers(0, d, 3)] = np.float32(np.nan)     # NaN keys rank above Inf: they are the top
    out["nans"] = n
    # one stretch a hundred times larger than the rest (a layer of another scale): every survivor
    # sits there, and the few waves that stream it may or may not have room for their lists
    w = rng.standard_normal(d).astype(np.float32)
    w[1_000_000:1_200_000] *= np.float32(100.0)
    out["one_loud_stretch"] = w
    return out


@pytest.mark.parametrize("inplace", [False, True])
def test_vectors_that_defeat_the_guess(inplace):
    d, k = 6_300_000 + 77, 6300
    rng = np.random.default_rng(77)
    zero = np.zeros(d, np.float32)
    gpu = FlatGpu(d, cap=k, inplace=inplace)
    expected = {"zeros": S.F_SHORTLIST_MISS, "constant": S.F_SHORTLIST_MISS,
                "small_ints": S.F_SHORTLIST_MISS, "sample_sees_zeros": S.F_SHORTLIST_MISS,
                "nans": S.F_SHORTLIST, "one_loud_stretch": None}
    for name, acc in defeating_vectors(d, rng).items():
        gpu.set_residual(zero)
        check_flat("topk", gpu, acc, zero, k, what=f"{name} inplace={inplace}")
        assert way(gpu) in (S.F_SHORTLIST, S.F_SHORTLIST_MISS)
        if expected[name] is not None:
            assert way(gpu) == expected[name], (name, inplace)


def test_the_lists_can_be_declined():
    """short_list = -1, the error norms, k beyond d/80 and a workspace of the smaller size all
    take the passes over acc from the start: same results, no way reported."""
    d, k = 6_100_000, 6100
    g = synth.normal(d, 41, 0, 0.01)
    eps = synth.normal(d, 42, 0, 0.003)
    gpu = FlatGpu(d, cap=d // 50)
    for kk, kw in ((k, {"short_list": -1}), (k, {"error_norms": True}), (d // 79, {})):
        gpu.set_residual(eps)
        check_flat("topk", gpu, g, eps, kk, what=f"{kw} k={kk}", **kw)
        assert way(gpu) == 0, (kk, kw)
    gpu.set_residual(eps)
    check_flat("topk", gpu, g, eps, d // 81, what="k = d/81")
    assert way(gpu) == S.F_SHORTLIST
    for tc in (1, 2, 5):
        gpu.set_residual(eps)
        check_flat("topk", gpu, g, eps, k, what=f"tile_chunks={tc}", tile_chunks=tc)
        assert way(gpu) == S.F_SHORTLIST, tc
    small = S.workspace_bytes_min(d, 1)
    assert small < gpu.b.workspace_nbytes
    gpu.b.workspace = torch.empty(small, dtype=torch.uint8, device="cuda:0")
    gpu.set_residual(eps)
    check_flat("topk", gpu, g, eps, k, what="small workspace")
    assert way(gpu) == 0


def test_a_call_with_lists_can_be_captured_in_a_hip_graph():
    """The way a call takes is decided on the device, so a captured call replays with or without
    the lists as each replay's data asks: typical gradients take them, an all-zero one does not."""
    from gpu_harness import same_bits
    from oracle import oracle as O
    d, k = 6_100_000, 6100
    b = S.Buffers.allocate(d, k)
    grad = torch.zeros(d, device="cuda:0")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):   # warm-up outside capture (first-call queries of the runtime)
        S.sparsify_topk(d, k, grad, b.residual, b.acc, b.out_idx, b.out_val, k, b.result, b.workspace,
                        b.workspace_nbytes)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        S.sparsify_topk(d, k, grad, b.residual, b.acc, b.out_idx, b.out_val, k, b.result, b.workspace,
                        b.workspace_nbytes)
    b.residual.zero_()
    eps = np.zeros(d, np.float32)
    for step in range(5):
        g = np.zeros(d, np.float32) if step == 2 else synth.normal(d, 77, step, 0.01)
        if step == 2:
            eps = np.zeros(d, np.float32)   # with a zero residual acc is all zero: no key above tau
            b.residual.zero_()
        grad.copy_(torch.from_numpy(g))
        b.out_idx.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        acc_o = O.accumulate(g, eps)
        idx_o, val_o, eps, ro = O.topk(acc_o, k)
        res = S.decode_results(b.result)[0]
        assert int(res["nnz"]) == k and int(res["topk_key"]) == ro.topk_key, step
        assert (int(res["flags"]) & S.F_WAY) == (S.F_SHORTLIST_MISS if step == 2 else S.F_SHORTLIST), step
        assert np.array_equal(b.out_idx[:k].cpu().numpy().view(np.uint32), idx_o), step
        assert same_bits(b.out_val[:k].cpu().numpy(), val_o), step
        assert same_bits(b.residual.cpu().numpy(), eps), step
        assert same_bits(b.acc.cpu().numpy(), acc_o), step
        _ = (b.acc * 2).sum().item()   # unrelated eager work between replays

"""Seeded random sweep of shapes, densities, value distributions, buffer modes and tilings for
the flat and the layer-wise calls, each case compared bit for bit with the oracle; plus two
compressors running concurrently on two streams, and the calibration copy."""
import numpy as np
import pytest
import torch

from gpu_harness import FlatGpu, SegGpu, check_flat, check_segmented, same_bits
from oracle import oracle as O
from paper_1911_08772_amd import sparsify as S
from paper_1911_08772_amd import synth

pytestmark = pytest.mark.gpu


def random_vector(rng, d, kind):
    if kind == 0:
        return (rng.standard_normal(d) * 10.0 ** rng.integers(-6, 3)).astype(np.float32)
    if kind == 1:
        return (rng.standard_t(2, d) * 1e-3).astype(np.float32)
    if kind == 2:
        return rng.integers(-5, 6, d).astype(np.float32)                      # ties everywhere
    if kind == 3:
        v = np.zeros(d, np.float32)                                           # sparse gradient
        n = max(1, d // 50)
        v[rng.integers(0, d, n)] = rng.standard_normal(n).astype(np.float32)
        return v
    return (rng.uniform(-1, 1, d) * (rng.uniform(0, 1, d) < 0.3)).astype(np.float32)


@pytest.mark.parametrize("selector", ["gaussiank", "topk", "dgck"])
def test_flat_random_cases(selector):
    rng = np.random.default_rng(20261127)
    for case in range(120):
        d = int(rng.choice([rng.integers(1, 300), rng.integers(300, 20_000), rng.integers(20_000, 600_000)]))
        k = int(rng.integers(1, max(2, d // int(rng.choice([1, 3, 30, 1000])) + 1)))
        k = min(max(k, 1), d)
        g = random_vector(rng, d, int(rng.integers(0, 5)))
        eps = random_vector(rng, d, int(rng.integers(0, 5))) if rng.random() < 0.7 else np.zeros(d, np.float32)
        inplace = bool(rng.random() < 0.4) and selector != "dgck"
        cap = d if selector != "gaussiank" or rng.random() < 0.5 else int(rng.integers(1, d + 1))
        cap = max(cap, k) if selector != "gaussiank" else cap
        kw = {"tile_chunks": int(rng.choice([0, 0, 1, 2, 3, 7]))}
        if selector == "dgck":
            kw["sample_stride"] = int(rng.choice([0, 1, 2, 10, 100, 333, 5000]))
            kw["sample_seed"] = int(rng.integers(0, 1 << 62))
        if selector == "gaussiank":
            kw["tail_div"] = float(rng.choice([2.0, 2.0, 1.0, 3.5]))
            kw["ddof"] = int(rng.choice([1, 1, 0]))
        gpu = FlatGpu(d, cap=cap, inplace=inplace)
        gpu.set_residual(eps)
        check_flat(selector, gpu, g, eps, k, what=f"case {case}: d={d} k={k} cap={cap} inplace={inplace} {kw}", **kw)


@pytest.mark.parametrize("selector", ["topk", "dgck", "gaussiank"])
def test_flat_random_cases_where_short_lists_are_built(selector):
    """From 6 M elements Top_k and DGC_k list the large entries in the accumulate pass and
    Gaussian_k in the count pass; whether a call ends up using its lists depends on the data,
    the results must not."""
    rng = np.random.default_rng(6_000_000 + len(selector))
    ways = set()
    for case in range(14):
        d = int(rng.integers(6_000_000, 11_000_000))
        k = int(rng.choice([1, rng.integers(2, 200), d // 1000, rng.integers(d // 500, d // 80)]))
        if selector == "gaussiank":
            g = awkward_vector(rng, d)
            eps = awkward_vector(rng, d) if rng.random() < 0.5 else np.zeros(d, np.float32)
        else:
            g = random_vector(rng, d, int(rng.integers(0, 5)))
            eps = random_vector(rng, d, int(rng.integers(0, 5))) if rng.random() < 0.6 else np.zeros(d, np.float32)
        inplace = bool(rng.random() < 0.4) and selector != "dgck"
        kw = {"tile_chunks": int(rng.choice([0, 0, 2, 5]))}
        if selector == "dgck":
            kw["sample_stride"] = int(rng.choice([0, 10, 37, 100, 1000, 5000]))
            kw["sample_seed"] = int(rng.integers(0, 1 << 62))
        if selector == "gaussiank":
            kw["tail_div"] = float(rng.choice([2.0, 2.0, 1.0]))
            kw["ddof"] = int(rng.choice([1, 0]))
        cap = k if selector != "gaussiank" else int(rng.choice([4 * k, d, max(1, k // 2)]))
        gpu = FlatGpu(d, cap=cap, inplace=inplace)
        gpu.set_residual(eps)
        check_flat(selector, gpu, g, eps, k, what=f"case {case}: d={d} k={k} inplace={inplace} {kw}", **kw)
        ways.add(int(S.decode_results(gpu.b.result)[0]["flags"]) & S.F_WAY)
        del gpu
    assert S.F_SHORTLIST in ways and ways <= {S.F_SHORTLIST, S.F_SHORTLIST_MISS}, ways


def awkward_vector(rng, d):
    """Bell-shaped, heavy-tailed, tied, sparse, uniform (no tail), two-level, one loud stretch, or
    far from zero: what makes Algorithm 1's walk end high, low or nowhere."""
    kind = int(rng.integers(0, 9))
    if kind < 5:
        return random_vector(rng, d, kind)
    if kind == 5:
        return rng.uniform(-1, 1, d).astype(np.float32)
    if kind == 6:
        v = (rng.standard_normal(d) * 1e-6).astype(np.float32)
        n = int(rng.integers(1, max(2, d // 50)))
        w = rng.choice(d, n, replace=False)
        v[w[: n // 3]] = 1.0
        v[w[n // 3:]] = np.float32(rng.uniform(0.01, 0.2))
        return v
    if kind == 7:
        v = rng.standard_normal(d).astype(np.float32)
        a = int(rng.integers(0, max(1, d - 300_000)))
        v[a:a + int(rng.integers(1000, 300_000))] *= np.float32(100)
        return v
    return (rng.standard_normal(d) * 0.01 + rng.choice([-5.0, 0.3, 5.0])).astype(np.float32)


@pytest.mark.parametrize("mode", [1, 0])
def test_segmented_random_cases_where_short_lists_are_built(mode):
    """Layer-wise calls on vectors of 6 M elements and more: every segment decides for itself
    whether its pairs come from its lists; results must not depend on it."""
    rng = np.random.default_rng(60_000_001 + mode)
    ways = set()
    for case in range(10):
        d = int(rng.integers(6_000_000, 8_500_000))
        L = int(rng.integers(2, 120))
        sizes = np.maximum(1, (rng.dirichlet(np.ones(L) * 0.3) * d).astype(np.int64))
        sizes[0] += d - int(sizes.sum())
        if sizes[0] < 1:
            continue
        seg_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
        seg_k = np.array([rng.integers(1, max(2, s // int(rng.choice([10, 100, 1000])) + 1)) for s in sizes], np.int64)
        seg_k = np.minimum(np.maximum(seg_k, 1), sizes)
        caps = np.array([max(4 * k, 16) if rng.random() < 0.8 else rng.integers(0, 2 * s + 2)
                         for s, k in zip(sizes, seg_k)], np.int64)
        g = np.concatenate([awkward_vector(rng, int(s)) if s > 400_000 else
                            random_vector(rng, int(s), int(rng.integers(0, 5))) for s in sizes])
        eps = awkward_vector(rng, d) if rng.random() < 0.4 else np.zeros(d, np.float32)
        gpu = SegGpu(seg_off, seg_k, caps, inplace=bool(rng.random() < 0.3))
        gpu.set_residual(eps)
        check_segmented(mode, gpu, g, eps, what=f"mode {mode} case {case}: L={L} d={d}", tile_chunks=int(rng.choice([0, 0, 1, 3])))
        ways |= {int(r["flags"]) & S.F_WAY for r in S.decode_results(gpu.b.result)
                 if not int(r["flags"]) & (S.F_BADSEGMENT | S.F_OVERFLOW)}
        del gpu
    # both ways were exercised (Top_k in place has no lists: no way bit at all)
    assert ways - {0} == {S.F_SHORTLIST, S.F_SHORTLIST_MISS} and (mode == 0 or 0 not in ways), ways


@pytest.mark.parametrize("mode", [0, 1])
def test_segmented_random_cases(mode):
    rng = np.random.default_rng(77 + mode)
    for case in range(40):
        L = int(rng.integers(1, 40))
        sizes = np.maximum(1, (10.0 ** rng.uniform(0, 4.7, L)).astype(np.int64))
        seg_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
        seg_k = np.array([rng.integers(1, max(2, s // int(rng.choice([1, 10, 100])) + 1)) for s in sizes], np.int64)
        seg_k = np.minimum(np.maximum(seg_k, 1), sizes)
        caps = np.array([rng.integers(0, 2 * s + 2) if rng.random() < 0.3 else max(4 * k, 16)
                         for s, k in zip(sizes, seg_k)], np.int64)
        d = int(seg_off[-1])
        g = np.concatenate([random_vector(rng, int(s), int(rng.integers(0, 5))) for s in sizes])
        eps = random_vector(rng, d, 0) if rng.random() < 0.5 else np.zeros(d, np.float32)
        gpu = SegGpu(seg_off, seg_k, caps, inplace=bool(rng.random() < 0.3))
        gpu.set_residual(eps)
        check_segmented(mode, gpu, g, eps, what=f"case {case}: L={L} d={d}",
                        tile_chunks=int(rng.choice([0, 1, 3])))


def test_two_compressors_on_two_streams():
    """Independent instances (own buffers and workspaces) may run concurrently."""
    wl = synth.workload("cfg1_resnet20")
    d, k, cap = wl.d, wl.k, 4 * wl.k
    gs = [wl.grad(0), wl.grad(1)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    bufs = [S.Buffers.allocate(d, cap) for _ in range(2)]
    grads = [torch.from_numpy(g).to("cuda:0") for g in gs]
    torch.cuda.synchronize()
    for rep in range(10):
        for b in bufs:
            b.residual.zero_()
        torch.cuda.synchronize()
        for i in range(2):
            fn = S.sparsify_gaussiank if (i + rep) % 2 == 0 else S.sparsify_topk
            fn(d, k, grads[i], bufs[i].residual, bufs[i].acc, bufs[i].out_idx, bufs[i].out_val, cap,
               bufs[i].result, bufs[i].workspace, bufs[i].workspace_nbytes, stream=streams[i])
        torch.cuda.synchronize()
        for i in range(2):
            want = (O.gaussiank(gs[i], k, cap=cap) if (i + rep) % 2 == 0 else O.topk(gs[i], k))[2]
            assert same_bits(bufs[i].residual.cpu().numpy(), want), (rep, i)


def test_calibration_copy():
    n = 1_000_000
    src = torch.randn(n, device="cuda:0")
    dst = torch.zeros(n, device="cuda:0")
    S.sparsify_calibration_copy(dst, src, n)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    assert S.sparsify_calibration_copy(dst, src, 3, check=False) == S.E_INVALID
    assert S.sparsify_calibration_copy(dst, dst, n, check=False) == S.E_INVALID


@pytest.mark.parametrize("selector", ["gaussiank", "topk", "dgck"])
def test_calls_can_be_captured_in_a_hip_graph(selector):
    """The library never synchronises, allocates or uses memset nodes, so a call can be captured
    once and replayed on new gradients; every replay is checked against the oracle chain, with
    eager work and synchronisations between the replays."""
    wl = synth.workload("cfg1_resnet20")
    d, k, cap = wl.d, wl.k, 4 * wl.k
    b = S.Buffers.allocate(d, cap)
    grad = torch.zeros(d, device="cuda:0")
    fn = {"gaussiank": S.sparsify_gaussiank, "topk": S.sparsify_topk, "dgck": S.sparsify_dgck}[selector]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):   # warm-up outside capture (first-call queries of the runtime)
        fn(d, k, grad, b.residual, b.acc, b.out_idx, b.out_val, cap, b.result, b.workspace,
           b.workspace_nbytes)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fn(d, k, grad, b.residual, b.acc, b.out_idx, b.out_val, cap, b.result, b.workspace,
           b.workspace_nbytes)
    b.residual.zero_()
    eps = np.zeros(d, np.float32)
    for step in range(6):
        g = wl.grad(step)
        grad.copy_(torch.from_numpy(g))
        b.out_idx.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        acc_o = O.accumulate(g, eps)
        idx_o, val_o, eps, ro = (O.gaussiank(acc_o, k, cap=cap) if selector == "gaussiank"
                                 else O.topk(acc_o, k) if selector == "topk" else O.dgck(acc_o, k))
        res = S.decode_results(b.result)[0]
        n = int(res["nnz"])
        assert n == ro.nnz
        gi = b.out_idx[:n].cpu().numpy().view(np.uint32)
        assert np.array_equal(np.sort(gi), idx_o), (selector, step)
        assert same_bits(b.residual.cpu().numpy(), eps), (selector, step)
        assert same_bits(b.acc.cpu().numpy(), acc_o), (selector, step)
        _ = (b.acc * 2).sum().item()   # unrelated eager work between replays

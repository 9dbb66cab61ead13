"""The entry point that allocates nothing (sparsify_gaussiank_static: workspace in an array built
into the library) against sparsify_gaussiank with a caller-owned workspace, through the C ABI:
record, pairs, acc and residual bit for bit, on two calls in a row, the second on a shorter
vector (the array then still holds the longer call's partial results)."""
import numpy as np
import pytest
import torch

from gpu_harness import DEV, same_bits
from paper_1911_08772_amd import sparsify as S
from paper_1911_08772_amd import synth

pytestmark = pytest.mark.gpu


def run_both(d, k, g, eps):
    cap = max(4 * k, 1024)
    out = []
    grad = torch.from_numpy(g).to(DEV)
    for static in (False, True):
        b = S.Buffers.allocate(d, cap, 1, False, DEV)
        b.residual.copy_(torch.from_numpy(eps))
        b.out_idx.fill_(-1)
        b.out_val.fill_(float("nan"))
        b.acc.fill_(float("nan"))
        if static:
            S.sparsify_gaussiank_static(d, k, grad, b.residual, b.acc, b.out_idx, b.out_val, cap,
                                        b.result)
        else:
            S.sparsify_gaussiank(d, k, grad, b.residual, b.acc, b.out_idx, b.out_val, cap,
                                 b.result, b.workspace, b.workspace_nbytes)
        torch.cuda.synchronize()
        out.append({"rec": b.result.cpu().numpy().copy(), "idx": b.out_idx.cpu().numpy(),
                    "val": b.out_val.cpu().numpy(), "acc": b.acc.cpu().numpy(),
                    "eps": b.residual.cpu().numpy()})
    return out


def test_static_workspace_call_equals_the_workspace_call_twice_in_a_row():
    seen = []
    #          long first (many tiles, three-chunk tiles), then short and ragged (one-chunk tiles)
    for d, k, seed in [(9_000_017, 9001, 31), (300_003, 301, 32)]:
        g = synth.normal(d, seed, 0, 1e-3)
        eps = synth.normal(d, seed, 1, 2e-3)
        ref, got = run_both(d, k, g, eps)
        rec = ref["rec"].view(S.RESULT_DTYPE)[0]
        rec["flags"] &= ~np.uint32(S.F_WAY)   # (which way the workspace call took is no result)
        assert int(rec["nnz"]) > 0 and int(rec["rounds"]) >= 1
        assert np.array_equal(ref["rec"], got["rec"]), (d, rec, got["rec"].view(S.RESULT_DTYPE)[0])
        assert np.array_equal(ref["idx"], got["idx"]), d      # same slots, nothing beyond nnz
        assert same_bits(ref["val"], got["val"]), d
        assert same_bits(ref["acc"], got["acc"]), d
        assert same_bits(ref["eps"], got["eps"]), d
        seen.append(int(rec["nnz"]))
    assert len(seen) == 2


def test_static_workspace_call_rejects_what_it_cannot_hold():
    t = torch.zeros(1024, dtype=torch.float32, device=DEV)
    big = S.STATIC_MAX_D + 1
    rc = S.sparsify_gaussiank_static(big, 10, t, t, t, t, t, 64, t, check=False)
    assert rc == S.E_WORKSPACE      # checked before any pointer is looked at or kernel launched
    rc = S.sparsify_gaussiank_static(1000, 0, t, t, t, t, t, 64, t, check=False)
    assert rc == S.E_INVALID

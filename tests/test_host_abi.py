"""Host-side checks that need no GPU: the C-ABI library loads, exports every function that
include/sparsify.h declares, sizes the workspace sensibly and rejects bad arguments before
launching anything."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_1911_08772_amd import sparsify as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "sparsify.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sparsify_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    names = declared_functions()
    assert set(names) == set(S.EXPORTS), (names, S.EXPORTS)
    for n in names:
        assert getattr(S.lib, n) is not None
    assert "gfx950" in S.version()


def test_result_record_layout_matches_header():
    assert S.RESULT_BYTES == 96
    assert S.RESULT_DTYPE.fields["mean"][1] == 32 and S.RESULT_DTYPE.fields["topk_key"][1] == 72
    assert S.RESULT_DTYPE.fields["acc_sqnorm"][1] == 80
    assert C.sizeof(S.Opts) == 48 and S.Opts.sample_seed.offset == 32 and S.Opts.short_list.offset == 40


def test_workspace_bytes():
    assert S.workspace_bytes(0, 1) == 0 and S.workspace_bytes(10, 0) == 0
    assert S.workspace_bytes(1 << 31, 1) == 0
    assert S.workspace_bytes_min(0, 1) == 0 and S.workspace_bytes_min(1 << 31, 1) == 0
    small, big = S.workspace_bytes_min(1000, 1), S.workspace_bytes_min(66_034_000, 1)
    assert 0 < small < big < 4 * 1024 * 1024
    assert S.workspace_bytes_min(25_557_032, 54) > S.workspace_bytes_min(25_557_032, 1)
    assert small % 256 == 0 and big % 256 == 0
    # the size to allocate adds the short lists for vectors of 6 M elements and more in up to
    # 1024 segments: 0.1 entries of 8 bytes per element and the per-run records (8 bytes per 256
    # elements, plus those of every segment's ragged first and last tile)
    for d, L in ((1000, 1), (5_999_999, 1), (5_999_999, 54), (25_557_032, 1025)):
        assert S.workspace_bytes(d, L) == S.workspace_bytes_min(d, L)
    for d in (6_000_000, 25_557_032, 66_034_000, 536_870_912):
        for L in (1, 54, 1024):
            extra = S.workspace_bytes(d, L) - S.workspace_bytes_min(d, L)
            assert 0.8 * d < extra < 0.9 * d + (3 << 20) + 8 * 16 * 40 * (2 * L + 1), (d, L, extra)
            assert S.workspace_bytes(d, L) % 256 == 0


BASE = 0x7000_0000_0000  # fake, 256-byte aligned "device" addresses; never dereferenced


def flat_args(d=1000, k=10, cap=64, **over):
    n = 4 * d
    a = dict(d=d, k=k, grad=BASE, residual=BASE + (1 << 32), acc=BASE + (2 << 32),
             out_idx=BASE + (3 << 32), out_val=BASE + (4 << 32), cap=cap,
             result=BASE + (5 << 32), workspace=BASE + (6 << 32),
             workspace_nbytes=S.workspace_bytes(max(d, 1), 1) if 0 < d < (1 << 31) else 1 << 20)
    a.update(over)
    return a, n


@pytest.mark.parametrize("fn", [S.sparsify_gaussiank, S.sparsify_topk, S.sparsify_dgck])
def test_flat_calls_reject_bad_arguments_before_any_launch(fn):
    def rc(**over):
        a, _ = flat_args(**over)
        return fn(a["d"], a["k"], a["grad"], a["residual"], a["acc"], a["out_idx"], a["out_val"],
                  a["cap"], a["result"], a["workspace"], a["workspace_nbytes"], stream=0,
                  check=False)
    assert rc(d=0) == S.E_INVALID
    assert rc(d=1 << 31) == S.E_INVALID
    assert rc(k=0) == S.E_INVALID
    assert rc(k=1001) == S.E_INVALID
    assert rc(cap=0) == S.E_INVALID
    assert rc(grad=0) == S.E_INVALID
    assert rc(result=0) == S.E_INVALID
    assert rc(grad=BASE + 4) == S.E_INVALID                       # misaligned
    assert rc(acc=BASE + 8) == S.E_INVALID                        # acc overlaps grad
    assert rc(residual=BASE + (2 << 32) + 16) == S.E_INVALID      # partial overlap acc/residual
    assert rc(out_val=BASE + (3 << 32)) == S.E_INVALID            # out_val == out_idx
    assert rc(workspace=0) == S.E_WORKSPACE
    assert rc(workspace=BASE + (6 << 32) + 64) == S.E_WORKSPACE   # misaligned workspace
    assert rc(workspace_nbytes=128) == S.E_WORKSPACE
    if fn is not S.sparsify_gaussiank:
        assert rc(k=100, cap=99) == S.E_INVALID                   # Top_k and DGC_k need cap >= k


def test_dgck_rejects_in_place_buffers_and_bad_sampling():
    a, _ = flat_args()
    common = (a["out_idx"], a["out_val"], a["cap"], a["result"], a["workspace"], a["workspace_nbytes"])
    assert S.sparsify_dgck(a["d"], a["k"], a["grad"], a["residual"], a["residual"], *common,
                           stream=0, check=False) == S.E_INVALID   # its key lists need the residual
    assert S.sparsify_dgck(a["d"], a["k"], a["grad"], a["residual"], a["acc"], *common,
                           sample_stride=-3, stream=0, check=False) == S.E_INVALID


def test_gaussiank_rejects_bad_options():
    a, _ = flat_args()
    for kw in (dict(tail_div=0.5), dict(tail_div=float("nan")), dict(ddof=2)):
        rc = S.sparsify_gaussiank(a["d"], a["k"], a["grad"], a["residual"], a["acc"], a["out_idx"],
                                  a["out_val"], a["cap"], a["result"], a["workspace"],
                                  a["workspace_nbytes"], stream=0, check=False, **kw)
        assert rc == S.E_INVALID


def test_segmented_rejects_bad_arguments():
    a, _ = flat_args()
    seg = BASE + (7 << 32)

    def rc(L=3, d=1000, mode=1, seg_off=seg, seg_k=seg + 4096, out_off=seg + 8192, **over):
        b = dict(a)
        b.update(over)
        return S.sparsify_segmented(L, d, seg_off, seg_k, mode, b["grad"], b["residual"], b["acc"],
                                    b["out_idx"], b["out_val"], out_off, b["cap"], b["result"],
                                    b["workspace"], S.workspace_bytes(1000, 3), stream=0,
                                    check=False)
    assert rc(L=0) == S.E_INVALID
    assert rc(mode=2) == S.E_INVALID
    assert rc(seg_off=0) == S.E_INVALID
    assert rc(seg_k=seg + 4) == S.E_INVALID
    assert rc(d=0) == S.E_INVALID
    assert rc(L=50) == S.E_WORKSPACE  # workspace sized for 3 segments


def test_static_workspace_call_rejects_long_vectors_before_anything_else():
    """The entry point without a workspace argument holds at most 2^27 elements' worth of partial
    results: a longer vector is refused on the host, before any device call."""
    a, _ = flat_args()
    rc = S.sparsify_gaussiank_static(S.STATIC_MAX_D + 1, 10, a["grad"], a["residual"], a["acc"],
                                     a["out_idx"], a["out_val"], a["cap"], a["result"], stream=0,
                                     check=False)
    assert rc == S.E_WORKSPACE
    assert S.workspace_bytes_min(S.STATIC_MAX_D, 1) <= 6 << 20 < S.workspace_bytes_min(2 * S.STATIC_MAX_D, 1)


def test_scatter_add_rejects_bad_arguments_before_any_launch():
    def rc(**over):
        a = dict(d=1000, P=4, idx=BASE, val=BASE + (1 << 32), stride=64, nnz=BASE + (2 << 32),
                 dense=BASE + (3 << 32), status=BASE + (4 << 32), nnz_stride_bytes=4)
        a.update(over)
        return S.sparsify_scatter_add(a["d"], a["P"], a["idx"], a["val"], a["stride"], a["nnz"],
                                      a["dense"], a["status"], nnz_stride_bytes=a["nnz_stride_bytes"],
                                      stream=0, check=False)
    assert rc(d=0) == S.E_INVALID and rc(d=1 << 31) == S.E_INVALID
    assert rc(P=0) == S.E_INVALID and rc(P=S.SCATTER_MAX_LISTS + 1) == S.E_INVALID
    assert rc(stride=0) == S.E_INVALID
    assert rc(idx=0) == S.E_INVALID and rc(val=0) == S.E_INVALID and rc(nnz=0) == S.E_INVALID
    assert rc(dense=0) == S.E_INVALID and rc(status=0) == S.E_INVALID
    assert rc(dense=BASE + (3 << 32) + 4) == S.E_INVALID          # dense must be 16-byte aligned
    assert rc(nnz_stride_bytes=0) == S.E_INVALID and rc(nnz_stride_bytes=6) == S.E_INVALID
    assert rc(dense=BASE + 64) == S.E_INVALID                     # dense overlaps the index lists
    assert rc(dense=BASE + (1 << 32)) == S.E_INVALID              # dense is the value buffer
    assert rc(status=BASE + (3 << 32) + 400) == S.E_INVALID       # status inside dense


def test_flat_calls_refuse_a_forced_tile_length_their_tables_cannot_hold():
    a, _ = flat_args(d=25_557_032, k=25_558, cap=25_558)
    def rc(fn, tc, inplace=False):
        acc = a["residual"] if inplace else a["acc"]
        return fn(a["d"], a["k"], a["grad"], a["residual"], acc, a["out_idx"], a["out_val"], a["cap"],
                  a["result"], a["workspace"], a["workspace_nbytes"], stream=0, check=False,
                  tile_chunks=tc)
    for fn in (S.sparsify_gaussiank, S.sparsify_topk, S.sparsify_dgck):
        assert rc(fn, 1) == S.E_INVALID      # 6240 one-chunk tiles, the group tables hold 4096
        assert rc(fn, -1) == S.E_INVALID
    assert rc(S.sparsify_gaussiank, 1, inplace=True) == S.E_INVALID
    assert rc(S.sparsify_topk, 1, inplace=True) == S.E_INVALID
    # beyond 123 M elements the tables of Gaussian_k and of Top_k with a separate acc hold 65536
    # tiles; those of Top_k in place still 4096
    big, _ = flat_args(d=200_000_000, k=200_000, cap=200_000)
    rc_big = S.sparsify_topk(big["d"], big["k"], big["grad"], big["residual"], big["residual"],
                             big["out_idx"], big["out_val"], big["cap"], big["result"], big["workspace"],
                             big["workspace_nbytes"], stream=0, check=False, tile_chunks=1)
    assert rc_big == S.E_INVALID         # 48829 one-chunk tiles

"""Shared plumbing of the GPU parity tests: run the HIP path through the C ABI on torch-owned
device buffers, fetch the outputs, and compare them with the CPU oracle's on the same host
inputs.  Bit-exact for acc, indices (in ascending order), values and residuals; thresholds within 1e-6 relative
(their moments are summed in a different order), counts/rounds/flags exactly equal."""
import math
import os
import time

import numpy as np
import torch

from oracle import oracle as O
from paper_1911_08772_amd import sparsify as S

DEV = "cuda:0"
THRES_RTOL = 1e-6


def progress(msg: str) -> None:
    """Long tests leave a trail for whoever watches the run from outside: one line per step,
    appended to the file named by SPARSIFY_TEST_PROGRESS (nothing if it is not set)."""
    path = os.environ.get("SPARSIFY_TEST_PROGRESS")
    if not path:
        return
    try:
        with open(path, "a") as f:
            f.write(f"{time.strftime('%H:%M:%S')} {msg}\n")
    except OSError:
        pass


class FlatGpu:
    """One flat compressor instance on the GPU: buffers persist, so the residual carries over
    successive `step` calls exactly as in Eq. (2)."""

    def __init__(self, d: int, cap: int, inplace: bool = False):
        self.d, self.cap, self.inplace = d, cap, inplace
        self.b = S.Buffers.allocate(d, cap, 1, inplace, DEV)
        self.grad = torch.empty(d, dtype=torch.float32, device=DEV)

    def set_residual(self, eps: np.ndarray) -> None:
        self.b.residual.copy_(torch.from_numpy(eps))

    def step(self, selector: str, g: np.ndarray, k: int, fetch_dense: bool = True, **kw):
        b = self.b
        self.grad.copy_(torch.from_numpy(g))
        b.out_idx.fill_(-1)
        b.out_val.fill_(float("nan"))
        if not self.inplace:
            b.acc.fill_(float("nan"))
        fn = {"gaussiank": S.sparsify_gaussiank, "topk": S.sparsify_topk,
              "dgck": S.sparsify_dgck}[selector]
        fn(self.d, k, self.grad, b.residual, b.acc, b.out_idx, b.out_val, self.cap, b.result,
           b.workspace, b.workspace_nbytes, **kw)
        torch.cuda.synchronize()
        res = S.decode_results(b.result)[0]
        nnz = int(res["nnz"])
        out = {"res": res, "idx": b.out_idx[:nnz].cpu().numpy().view(np.uint32),
               "val": b.out_val[:nnz].cpu().numpy(),
               "tail_idx": b.out_idx[nnz:nnz + 8].cpu().numpy()}
        if fetch_dense:
            out["eps"] = b.residual.cpu().numpy()
            out["acc"] = None if self.inplace else b.acc.cpu().numpy()
        return out


def same_bits(a: np.ndarray, b: np.ndarray) -> bool:
    return a.shape == b.shape and np.array_equal(a.view(np.uint32), b.view(np.uint32))


def assert_pairs_match(got, idx_o, val_o, what=""):
    """Indices and values bit-exact, in the oracle's order: ascending index, as every selector of
    the library promises."""
    gi, gv = got["idx"], got["val"]
    assert gi.size == idx_o.size, (what, gi.size, idx_o.size)
    assert np.array_equal(gi, idx_o), what
    assert same_bits(gv, val_o), what
    assert np.all(got["tail_idx"] == -1), what  # nothing written beyond nnz


def assert_same_threshold(res, ro: O.Result, acc=None, what=""):
    """The fp32 threshold the final mask compared against.  GPU and oracle sum the moments in
    fp64 in different orders, so their fp64 thresholds differ in the last bits (the oracle's
    plain running sums over d entries are themselves within d * 2^-53 relative of the exact
    moments, the bound this check allows twice: 2e-11 was seen on a heavy-tailed vector of 6.9 M
    entries, where the kernels' partial sums matched extended precision to 4e-16; far inside the
    1e-6 the benchmark spec allows) and can, once in thousands of vectors, round to neighbouring
    fp32 values.  That is accepted when no entry of `acc` lies between the two (both thresholds
    then select the same entries, which the callers go on to compare bit for bit); otherwise the
    bits must be equal."""
    g32, o32 = np.float32(res["thres_f32"]), np.float32(ro.thres_f32)
    if g32.view(np.uint32) == o32.view(np.uint32):
        return
    assert acc is not None and np.isfinite(g32) and np.isfinite(o32), (what, g32, o32)
    rtol = max(1e-11, 2.0 * acc.size * 2.0 ** -53)
    assert abs(float(res["thres"]) - ro.thres) <= rtol * abs(ro.thres), (what, res["thres"], ro.thres)
    lo, hi = min(g32, o32), max(g32, o32)
    assert np.nextafter(lo, np.float32(np.inf)) == hi, (what, g32, o32)   # neighbours
    m = np.abs(acc)
    assert not np.any((m > lo) & (m <= hi)), (what, g32, o32)


def assert_gaussiank_result(res, ro: O.Result, what="", acc=None):
    assert int(res["rounds"]) == ro.rounds, (what, res, ro)
    assert list(res["count"]) == list(ro.count), (what, res, ro)
    assert int(res["flags"]) & ~S.F_WAY == ro.flags, (what, res, ro)  # (the way taken is no result)
    assert int(res["nnz"]) == ro.nnz, (what, res, ro)
    for name in ("mean", "std", "z", "thres0", "thres"):
        g, o = float(res[name]), getattr(ro, name)
        if (ro.flags & O.F_NONFINITE) and name in ("mean", "std"):
            continue  # Inf/NaN input: which non-finite value the moments take is not specified
        if math.isnan(o):
            assert math.isnan(g), (what, name, g, o)
        elif name == "mean":
            assert abs(g - o) <= 1e-9 * max(abs(o), ro.std, 1e-300), (what, name, g, o)
        else:
            assert g == o or abs(g - o) <= THRES_RTOL * abs(o), (what, name, g, o)
    assert_same_threshold(res, ro, acc, what)
    assert int(res["topk_key"]) == 0 and int(res["topk_ties_taken"]) == 0


def assert_topk_result(res, ro: O.Result, what=""):
    assert int(res["nnz"]) == ro.nnz, (what, res, ro)
    assert int(res["topk_key"]) == ro.topk_key, (what, res, ro)
    assert int(res["topk_ties_taken"]) == ro.topk_ties_taken, (what, res, ro)
    assert int(res["rounds"]) == 0 and int(res["flags"]) & ~S.F_WAY == 0, (what, res)  # (the way taken is no result)


def assert_dgck_result(res, ro: O.Result, what=""):
    for name in ("nnz", "rounds", "topk_key", "topk_ties_taken"):
        assert int(res[name]) == getattr(ro, name), (what, name, res, ro)
    assert int(res["flags"]) & ~S.F_WAY == ro.flags, (what, res, ro)  # (the way taken is no result)
    assert tuple(int(c) for c in res["count"]) == tuple(ro.count), (what, res, ro)
    g32, o32 = np.float32(res["thres_f32"]), np.float32(ro.thres_f32)
    assert g32.view(np.uint32) == o32.view(np.uint32), (what, g32, o32)
    assert float(res["thres"]) == ro.thres or (math.isnan(ro.thres) and math.isnan(float(res["thres"])))


def check_flat(selector, gpu: FlatGpu, g, eps_in, k, what="", **kw):
    """One step on both sides from the same (g, eps_in); returns the oracle's eps'."""
    acc_o = O.accumulate(g, eps_in)
    got = gpu.step(selector, g, k, **kw)
    if selector == "gaussiank":
        idx_o, val_o, eps_o, ro = O.gaussiank(acc_o, k, cap=gpu.cap,
                                              tail_div=kw.get("tail_div", 2.0),
                                              ddof=kw.get("ddof", 1))
        assert_gaussiank_result(got["res"], ro, what, acc=acc_o)
    elif selector == "dgck":
        idx_o, val_o, eps_o, ro = O.dgck(acc_o, k, kw.get("sample_stride", 0) or 100,
                                         kw.get("sample_seed", 0))
        assert_dgck_result(got["res"], ro, what)
        assert np.all(np.diff(got["idx"].astype(np.int64)) > 0), what  # ascending index order
    else:
        idx_o, val_o, eps_o, ro = O.topk(acc_o, k)
        assert_topk_result(got["res"], ro, what)
    if got["acc"] is not None:
        assert same_bits(got["acc"], acc_o), what
    assert_pairs_match(got, idx_o, val_o, what)
    assert same_bits(got["eps"], eps_o), what
    return eps_o


class SegGpu:
    """One layer-wise compressor instance: layout arrays resident on the device."""

    def __init__(self, seg_off: np.ndarray, seg_k: np.ndarray, caps: np.ndarray,
                 inplace: bool = False):
        self.L = int(seg_k.size)
        self.d = int(seg_off[-1])
        self.seg_off, self.seg_k = seg_off.astype(np.int64), seg_k.astype(np.int64)
        self.out_off = np.concatenate([[0], np.cumsum(caps)]).astype(np.int64)
        self.out_cap = max(int(self.out_off[-1]), 1)
        self.inplace = inplace
        self.b = S.Buffers.allocate(self.d, self.out_cap, self.L, inplace, DEV)
        self.grad = torch.empty(self.d, dtype=torch.float32, device=DEV)
        self.d_seg_off = torch.from_numpy(self.seg_off).to(DEV)
        self.d_seg_k = torch.from_numpy(self.seg_k).to(DEV)
        self.d_out_off = torch.from_numpy(self.out_off).to(DEV)

    def set_residual(self, eps: np.ndarray) -> None:
        self.b.residual.copy_(torch.from_numpy(eps))

    def step(self, mode: int, g: np.ndarray, **kw):
        b = self.b
        self.grad.copy_(torch.from_numpy(g))
        b.out_idx.fill_(-1)
        b.out_val.fill_(float("nan"))
        S.sparsify_segmented(self.L, self.d, self.d_seg_off, self.d_seg_k, mode, self.grad,
                             b.residual, b.acc, b.out_idx, b.out_val, self.d_out_off, self.out_cap,
                             b.result, b.workspace, b.workspace_nbytes, **kw)
        torch.cuda.synchronize()
        return {"res": S.decode_results(b.result), "idx": b.out_idx.cpu().numpy(),
                "val": b.out_val.cpu().numpy(), "eps": b.residual.cpu().numpy(),
                "acc": None if self.inplace else b.acc.cpu().numpy()}


def check_segmented(mode: int, gpu: SegGpu, g, eps_in, what="", **kw):
    acc_o = O.accumulate(g, eps_in)
    got = gpu.step(mode, g, **kw)
    idx_o, val_o, eps_o, res_o = O.segmented(acc_o, gpu.seg_off, gpu.seg_k, mode, gpu.out_off,
                                             tail_div=kw.get("tail_div", 2.0),
                                             ddof=kw.get("ddof", 1))
    if got["acc"] is not None:
        assert same_bits(got["acc"], acc_o), what
    for l in range(gpu.L):
        w = f"{what} segment {l}"
        res, ro = got["res"][l], res_o[l]
        if mode == 1:
            assert_gaussiank_result(res, ro, w, acc=acc_o[int(gpu.seg_off[l]):int(gpu.seg_off[l + 1])])
        else:
            assert int(res["nnz"]) == ro.nnz and int(res["flags"]) & ~S.F_WAY == ro.flags, (w, res, ro)  # (the way taken is no result)
            assert int(res["topk_key"]) == ro.topk_key, (w, res, ro)
            assert int(res["topk_ties_taken"]) == ro.topk_ties_taken, (w, res, ro)
        o0, o1, n = int(gpu.out_off[l]), int(gpu.out_off[l + 1]), ro.nnz
        gi, gv = got["idx"][o0:o0 + n].view(np.uint32), got["val"][o0:o0 + n]
        assert np.array_equal(gi, idx_o[o0:o0 + n]), w       # ascending index inside the segment
        assert same_bits(gv, val_o[o0:o0 + n]), w
        assert np.all(got["idx"][o0 + n:o1] == -1), w  # nothing beyond nnz in this range
    assert same_bits(got["eps"], eps_o), what
    return eps_o

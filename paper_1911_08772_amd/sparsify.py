"""Python face of libsparsify.so (include/sparsify.h): argument marshalling only.

Every step of the compressor runs in the HIP kernels behind the C ABI; this module turns torch
tensors into device pointers, passes the current HIP stream, and decodes the result records.
PyTorch is used for device memory and streams only.  There is no CPU fallback: if the library
cannot be loaded the import of this module fails.
"""
import ctypes as C
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

from . import build as _build

OK, E_INVALID, E_WORKSPACE, E_LAUNCH = 0, 1, 2, 3
F_OVERFLOW, F_NONFINITE, F_EXHAUSTED, F_BADSEGMENT = 1, 2, 4, 8
F_SHORTLIST, F_SHORTLIST_MISS = 16, 32      # which way a flat Top_k call took, not a result
F_WAY = F_SHORTLIST | F_SHORTLIST_MISS

RESULT_DTYPE = np.dtype([("nnz", "<u4"), ("rounds", "<u4"), ("count", "<u4", (4,)),
                         ("flags", "<u4"), ("thres_f32", "<f4"), ("mean", "<f8"), ("std", "<f8"),
                         ("z", "<f8"), ("thres0", "<f8"), ("thres", "<f8"), ("topk_key", "<u4"),
                         ("topk_ties_taken", "<u4"), ("acc_sqnorm", "<f8"),
                         ("residual_sqnorm", "<f8")])
RESULT_BYTES = RESULT_DTYPE.itemsize  # 96


class Opts(C.Structure):
    _fields_ = [("tail_div", C.c_double), ("ddof", C.c_int32), ("tile_chunks", C.c_int32),
                ("trace", C.c_void_p), ("error_norms", C.c_int32), ("sample_stride", C.c_int32),
                ("sample_seed", C.c_uint64), ("short_list", C.c_int32)]


_p = C.c_void_p
lib = C.CDLL(_build.ensure_sparsify())
lib.sparsify_version.restype = C.c_char_p
lib.sparsify_workspace_bytes.argtypes = [C.c_int64, C.c_int32]
lib.sparsify_workspace_bytes.restype = C.c_size_t
lib.sparsify_workspace_bytes_min.argtypes = [C.c_int64, C.c_int32]
lib.sparsify_workspace_bytes_min.restype = C.c_size_t
_flat = [C.c_int64, C.c_int64, _p, _p, _p, _p, _p, C.c_int64, _p, _p, C.c_size_t,
         C.POINTER(Opts), _p]
lib.sparsify_gaussiank.argtypes = _flat
lib.sparsify_topk.argtypes = _flat
lib.sparsify_dgck.argtypes = _flat
lib.sparsify_gaussiank_static.argtypes = [C.c_int64, C.c_int64, _p, _p, _p, _p, _p, C.c_int64, _p,
                                          C.POINTER(Opts), _p]
lib.sparsify_segmented.argtypes = [C.c_int32, C.c_int64, _p, _p, C.c_int32, _p, _p, _p, _p, _p,
                                   _p, C.c_int64, _p, _p, C.c_size_t, C.POINTER(Opts), _p]
lib.sparsify_scatter_add.argtypes = [C.c_int64, C.c_int32, _p, _p, C.c_int64, _p, C.c_int64,
                                     C.c_float, _p, _p, _p]
lib.sparsify_calibration_copy.argtypes = [_p, _p, C.c_int64, _p]
lib.sparsify_trace_create.restype = _p
lib.sparsify_trace_destroy.argtypes = [_p]
lib.sparsify_trace_destroy.restype = None
lib.sparsify_trace_num_stages.argtypes = [_p]
lib.sparsify_trace_stage_name.argtypes = [_p, C.c_int32]
lib.sparsify_trace_stage_name.restype = C.c_char_p
lib.sparsify_trace_stage_ms.argtypes = [_p, C.c_int32, C.POINTER(C.c_float)]

EXPORTS = ["sparsify_version", "sparsify_workspace_bytes", "sparsify_workspace_bytes_min", "sparsify_gaussiank", "sparsify_topk",
           "sparsify_dgck", "sparsify_gaussiank_static", "sparsify_scatter_add",
           "sparsify_segmented", "sparsify_calibration_copy", "sparsify_trace_create", "sparsify_trace_destroy",
           "sparsify_trace_num_stages", "sparsify_trace_stage_name", "sparsify_trace_stage_ms"]


class SparsifyError(RuntimeError):
    def __init__(self, status: int, where: str):
        names = {1: "SPARSIFY_E_INVALID", 2: "SPARSIFY_E_WORKSPACE", 3: "SPARSIFY_E_LAUNCH"}
        super().__init__(f"{where}: {names.get(status, status)}")
        self.status = status


def _ptr(t) -> int:
    """Device pointer of a torch tensor (or a raw integer address / None)."""
    if t is None:
        return 0
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _opts(tail_div: float, ddof: int, trace, tile_chunks: int = 0, error_norms: bool = False,
          sample_stride: int = 0, sample_seed: int = 0, short_list: int = 0) -> Opts:
    return Opts(float(tail_div), int(ddof), int(tile_chunks),
                trace.handle if trace is not None else None, 1 if error_norms else 0,
                int(sample_stride), int(sample_seed), int(short_list))


def version() -> str:
    return lib.sparsify_version().decode()


def workspace_bytes(d_total: int, num_segments: int = 1) -> int:
    return int(lib.sparsify_workspace_bytes(d_total, num_segments))


def workspace_bytes_min(d_total: int, num_segments: int = 1) -> int:
    return int(lib.sparsify_workspace_bytes_min(d_total, num_segments))


class Trace:
    """Per-kernel timings of one call (HIP events owned by the library)."""

    def __init__(self):
        self.handle = lib.sparsify_trace_create()
        if not self.handle:
            raise RuntimeError("sparsify_trace_create failed")

    def stages(self):
        """[(kernel name, milliseconds)] of the last traced call; sync the stream first."""
        out = []
        for i in range(lib.sparsify_trace_num_stages(self.handle)):
            ms = C.c_float()
            rc = lib.sparsify_trace_stage_ms(self.handle, i, C.byref(ms))
            if rc != OK:
                raise SparsifyError(rc, "sparsify_trace_stage_ms")
            out.append((lib.sparsify_trace_stage_name(self.handle, i).decode(), ms.value))
        return out

    def __del__(self):
        if getattr(self, "handle", None) and lib is not None:  # lib is gone at interpreter exit
            lib.sparsify_trace_destroy(self.handle)
            self.handle = None


def sparsify_gaussiank(d, k, grad, residual, acc, out_idx, out_val, cap, result, workspace,
                       workspace_nbytes, tail_div=2.0, ddof=1, trace=None, stream=None,
                       check=True, tile_chunks=0, error_norms=False, short_list=0) -> int:
    o = _opts(tail_div, ddof, trace, tile_chunks, error_norms, short_list=short_list)
    rc = lib.sparsify_gaussiank(d, k, _ptr(grad), _ptr(residual), _ptr(acc), _ptr(out_idx),
                                _ptr(out_val), cap, _ptr(result), _ptr(workspace),
                                workspace_nbytes, C.byref(o), _stream(stream))
    if check and rc != OK:
        raise SparsifyError(rc, "sparsify_gaussiank")
    return rc


STATIC_MAX_D = 1 << 27


def sparsify_gaussiank_static(d, k, grad, residual, acc, out_idx, out_val, cap, result,
                              tail_div=2.0, ddof=1, trace=None, stream=None, check=True,
                              tile_chunks=0, error_norms=False) -> int:
    """sparsify_gaussiank on the library's built-in workspace (d <= STATIC_MAX_D)."""
    o = _opts(tail_div, ddof, trace, tile_chunks, error_norms)
    rc = lib.sparsify_gaussiank_static(d, k, _ptr(grad), _ptr(residual), _ptr(acc), _ptr(out_idx),
                                       _ptr(out_val), cap, _ptr(result), C.byref(o),
                                       _stream(stream))
    if check and rc != OK:
        raise SparsifyError(rc, "sparsify_gaussiank_static")
    return rc


def sparsify_dgck(d, k, grad, residual, acc, out_idx, out_val, cap, result, workspace,
                  workspace_nbytes, sample_stride=0, sample_seed=0, trace=None, stream=None,
                  check=True, tile_chunks=0, error_norms=False, short_list=0) -> int:
    o = _opts(2.0, 1, trace, tile_chunks, error_norms, sample_stride, sample_seed, short_list)
    rc = lib.sparsify_dgck(d, k, _ptr(grad), _ptr(residual), _ptr(acc), _ptr(out_idx),
                           _ptr(out_val), cap, _ptr(result), _ptr(workspace), workspace_nbytes,
                           C.byref(o), _stream(stream))
    if check and rc != OK:
        raise SparsifyError(rc, "sparsify_dgck")
    return rc


def sparsify_topk(d, k, grad, residual, acc, out_idx, out_val, cap, result, workspace,
                  workspace_nbytes, trace=None, stream=None, check=True, tile_chunks=0,
                  error_norms=False, short_list=0) -> int:
    o = _opts(2.0, 1, trace, tile_chunks, error_norms, short_list=short_list)
    rc = lib.sparsify_topk(d, k, _ptr(grad), _ptr(residual), _ptr(acc), _ptr(out_idx),
                           _ptr(out_val), cap, _ptr(result), _ptr(workspace), workspace_nbytes,
                           C.byref(o), _stream(stream))
    if check and rc != OK:
        raise SparsifyError(rc, "sparsify_topk")
    return rc


def sparsify_segmented(num_segments, d_total, seg_off, seg_k, mode, grad, residual, acc, out_idx,
                       out_val, out_off, out_cap, results, workspace, workspace_nbytes,
                       tail_div=2.0, ddof=1, trace=None, stream=None, check=True,
                       tile_chunks=0, error_norms=False, short_list=0) -> int:
    o = _opts(tail_div, ddof, trace, tile_chunks, error_norms, short_list=short_list)
    rc = lib.sparsify_segmented(num_segments, d_total, _ptr(seg_off), _ptr(seg_k), mode,
                                _ptr(grad), _ptr(residual), _ptr(acc), _ptr(out_idx),
                                _ptr(out_val), _ptr(out_off), out_cap, _ptr(results),
                                _ptr(workspace), workspace_nbytes, C.byref(o), _stream(stream))
    if check and rc != OK:
        raise SparsifyError(rc, "sparsify_segmented")
    return rc


SCATTER_F_BAD_LIST, SCATTER_F_BAD_COUNT = 1, 2
SCATTER_MAX_LISTS = 1024


def sparsify_scatter_add(d, num_lists, idx, val, list_stride, nnz, dense, status, scale=1.0,
                         nnz_stride_bytes=4, stream=None, check=True) -> int:
    """dense = scale * sum over the lists; `nnz` may point into an array of result records
    (nnz_stride_bytes = RESULT_BYTES)."""
    rc = lib.sparsify_scatter_add(d, num_lists, _ptr(idx), _ptr(val), list_stride, _ptr(nnz),
                                  nnz_stride_bytes, float(scale), _ptr(dense), _ptr(status),
                                  _stream(stream))
    if check and rc != OK:
        raise SparsifyError(rc, "sparsify_scatter_add")
    return rc


def sparsify_calibration_copy(dst, src, n, stream=None, check=True) -> int:
    rc = lib.sparsify_calibration_copy(_ptr(dst), _ptr(src), n, _stream(stream))
    if check and rc != OK:
        raise SparsifyError(rc, "sparsify_calibration_copy")
    return rc


def decode_results(result_tensor) -> np.ndarray:
    """Device result records -> numpy structured array (synchronises through the copy)."""
    return result_tensor.cpu().numpy().view(RESULT_DTYPE)


@dataclass
class Buffers:
    """Device buffers of one compressor instance (allocation only; torch owns the memory)."""
    d: int
    num_segments: int
    cap: int
    residual: "object"
    acc: "object"
    out_idx: "object"
    out_val: "object"
    result: "object"
    workspace: "object"

    @property
    def workspace_nbytes(self) -> int:
        return self.workspace.numel()

    @staticmethod
    def allocate(d: int, cap: int, num_segments: int = 1, inplace: bool = False,
                 device: str = "cuda:0") -> "Buffers":
        import torch
        residual = torch.zeros(d, dtype=torch.float32, device=device)
        acc = residual if inplace else torch.empty(d, dtype=torch.float32, device=device)
        return Buffers(d, num_segments, cap, residual, acc,
                       torch.zeros(cap, dtype=torch.int32, device=device),
                       torch.zeros(cap, dtype=torch.float32, device=device),
                       torch.zeros(RESULT_BYTES * num_segments, dtype=torch.uint8, device=device),
                       torch.empty(workspace_bytes(d, num_segments), dtype=torch.uint8,
                                   device=device))

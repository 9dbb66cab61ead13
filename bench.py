"""Headline benchmark: Gaussian_k (and exact Top_k) sparsification of a ResNet-50-sized fp32
gradient vector (d = 25,557,032, rho = 0.001) on one MI355X.

One step = one pass of the whole hot path on a fresh synthetic gradient already resident in
HBM: accumulate, select (Algorithm 1), compact, residual, with the residual carried from step
to step as in Eq. (2).  `value` is algorithmic GB/s of the Gaussian_k path: the method's 24 B
per element (accumulate 12, one count pass 4, compaction 8; the figure the target is stated in)
+ 8 B per survivor, over the time.  What the kernels as run move is given beside it
(`bytes_per_elem_moved`, `GBps_moved`): 20 B per element when the short lists serve, which the
result records say (the count kernel also writes the residual, the compaction reads the lists).
The exact Top_k path, timed the same way, is reported on the bytes it moves (16 B per element
with its short lists, 24 without), and under
`also`: the same two selectors on the workloads that do not fit the last-level cache (LSTM-sized,
66 M elements) or sit below the headline (VGG-16-sized), in place, layer-wise, the sampling
comparator DGC_k, and the aggregation of 16 workers' lists (sparsify_scatter_add).

Prints ONE JSON line.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
# algorithmic bytes per element of each streaming kernel (fp32 reads/writes the method needs)
KERNEL_BYTES_PER_ELEM = {"accum_moments": 12, "gk_count": 4, "gk_compact": 8,
                         "topk_accum_hist": 12, "topk_filter": 4, "topk_compact": 8,
                         "topk_hist1": 4, "topk_hist2": 4, "topk_hist3": 4}
GK_BYTES_PER_ELEM = 24   # r g, r eps, w acc | r acc (one count pass) | r acc, w eps'
# Gaussian_k with short lists built in the count pass (from 6 M elements, when the lists serve:
# the result record says so): r g, r eps, w acc | r acc, w eps'; the compact kernel reads the
# lists (about k entries), not counted.  In place: r g, r eps, w acc | r acc.
GK_LIST_BYTES_PER_ELEM = 20
GK_LIST_INPLACE_BYTES_PER_ELEM = 16
# r g, r eps, w acc (+digit 1) | r acc (filter: candidates written out) | r acc, w eps'; the
# candidate lists the three later digit passes read are data dependent and not counted
TOPK_BYTES_PER_ELEM = 24
# Top_k with short lists built in the accumulate pass (from 6 M elements, when the lists serve:
# the result record says so): r g, r eps, w acc, w eps'; the lists, a fraction of a per cent of
# the vector, are not counted.  In place: r g, r eps, w acc.
TOPK_LIST_BYTES_PER_ELEM = 16
TOPK_LIST_INPLACE_BYTES_PER_ELEM = 12
GK_INPLACE_BYTES_PER_ELEM = 20   # the compaction pass only reads acc (and zeroes the survivors)
TOPK_INPLACE_BYTES_PER_ELEM = 28  # no room for candidates: 12 + 3 full digit passes + r acc


class StageMeans(dict):
    """Average duration per kernel over the traced steps; `.median` holds the medians (an
    interval between two events also contains whatever kept the host from enqueueing the next
    launch in time, so a single late step can lift an average)."""
    median = {}
    listed = 0.0


class Flat:
    """One flat compressor instance on a pool of gradients resident in HBM (step s uses gradient
    s modulo the pool size): timed chains and traced chains of W warm-up + K steps."""

    def __init__(self, S, torch, wl, grads, K, W, inplace=False, tile_chunks=0, short_list=0):
        self.S, self.torch, self.wl, self.grads, self.K, self.W = S, torch, wl, grads, K, W
        self.short_list = short_list
        self.d, self.k = wl.d, wl.k
        self.cap = max(4 * wl.k, 1024)
        self.tile_chunks = tile_chunks
        self.b = S.Buffers.allocate(wl.d, self.cap, 1, inplace, "cuda:0")
        self.stream = torch.cuda.current_stream()

    def run(self, fn, s, trace=None, result=None):
        b = self.b
        kw = {"short_list": self.short_list} if fn is self.S.sparsify_topk else {}
        fn(self.d, self.k, self.grads[s % len(self.grads)], b.residual, b.acc, b.out_idx, b.out_val,
           self.cap, b.result if result is None else result, b.workspace, b.workspace_nbytes,
           trace=trace, stream=self.stream, tile_chunks=self.tile_chunks, **kw)

    def timed(self, fn):
        """W warm-up steps then exactly K timed steps, bracketed by synchronisations; returns
        (ms per step, wall ms per step, event ms per step)."""
        torch, K, W = self.torch, self.K, self.W
        self.b.residual.zero_()
        for s in range(W):
            self.run(fn, s)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(self.stream)
        for s in range(W, W + K):
            self.run(fn, s)
        e1.record(self.stream)
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        return max(wall_ms, e0.elapsed_time(e1)) / K, wall_ms / K, e0.elapsed_time(e1) / K

    def traced(self, fn):
        """The same chain again, back to back as in the timed run, with a HIP event on the stream
        after every kernel (one trace and one result record per step, read after one final
        synchronisation): average duration per kernel, nnz and rounds per step."""
        S, torch, K, W = self.S, self.torch, self.K, self.W
        traces = [S.Trace() for _ in range(K)]
        records = torch.zeros((K, S.RESULT_BYTES), dtype=torch.uint8, device="cuda:0")
        self.b.residual.zero_()
        for s in range(W):
            self.run(fn, s)
        for i in range(K):
            self.run(fn, W + i, trace=traces[i], result=records[i])
        self.stream.synchronize()
        per, nnz, rounds, listed = {}, [], [], 0
        for i in range(K):
            for name, ms in traces[i].stages():
                per.setdefault(name, []).append(ms)
            r = S.decode_results(records[i])[0]
            nnz.append(int(r["nnz"]))
            rounds.append(int(r["rounds"]))
            listed += 1 if int(r["flags"]) & S.F_SHORTLIST else 0
        stage = StageMeans({n: sum(v) / len(v) for n, v in per.items()})
        stage.median = {n: statistics.median(v) for n, v in per.items()}
        stage.listed = listed / K   # share of the steps whose pairs came from the short lists (Top_k, DGC_k)
        return stage, nnz, rounds

    def spread(self, fn, repeats):
        """The timed chain `repeats` more times: min and median of ms per step."""
        xs = [self.timed(fn)[0] for _ in range(repeats)]
        return {"repeats": repeats, "min_ms": round(min(xs), 5),
                "median_ms": round(statistics.median(xs), 5), "max_ms": round(max(xs), 5)}


def park_gradients(torch, wl, n):
    """n fresh gradients of the workload, generated on the host and parked in HBM."""
    import numpy as np
    host = np.empty(wl.d, np.float32)
    grads = [torch.empty(wl.d, dtype=torch.float32, device="cuda:0") for _ in range(n)]
    for s in range(n):
        wl.grad(s, out=host)
        grads[s].copy_(torch.from_numpy(host))
    torch.cuda.synchronize()
    return grads


def gbps(bytes_per_elem, d, nnz_mean, ms):
    return (bytes_per_elem * d + 8.0 * nnz_mean) / (ms * 1e-3) / 1e9


def gk_bytes_per_elem(listed, inplace):
    """Algorithmic bytes per element of the Gaussian_k path as run: `listed` of the steps took
    the short-list way (20 B, 16 in place), the others three passes (24 B, 20 in place)."""
    a = GK_LIST_INPLACE_BYTES_PER_ELEM if inplace else GK_LIST_BYTES_PER_ELEM
    b = GK_INPLACE_BYTES_PER_ELEM if inplace else GK_BYTES_PER_ELEM
    return round(listed * a + (1.0 - listed) * b, 3)


def topk_bytes_per_elem(listed, inplace):
    """Algorithmic bytes per element of the Top_k path as run: `listed` of the steps took the
    short-list way (16 B, 12 in place), the others the passes over acc (24 B, 28 in place)."""
    a = TOPK_LIST_INPLACE_BYTES_PER_ELEM if inplace else TOPK_LIST_BYTES_PER_ELEM
    b = TOPK_INPLACE_BYTES_PER_ELEM if inplace else TOPK_BYTES_PER_ELEM
    return round(listed * a + (1.0 - listed) * b, 3)


def dominant(stage, d, inplace=False):
    """The streaming kernel with the longest average duration and its algorithmic GB/s."""
    per = dict(KERNEL_BYTES_PER_ELEM)
    if stage.listed == 1.0 and "gk_count" in stage:
        # with lists the count kernel also writes eps' and the compact kernel streams nothing
        per["gk_count"] = 4 if inplace else 8
        per["gk_compact"] = 0
    dom = max((n for n in stage if per.get(n, 0) > 0), key=lambda n: stage[n])
    nbytes = per[dom] * d
    return dom, nbytes, nbytes / (stage[dom] * 1e-3) / 1e9


def side_workload(S, torch, synth, name, K, W):
    """Gaussian_k and Top_k on another workload: the same K steps after W warm-up steps, one
    fresh gradient per step."""
    import numpy as np
    wl = synth.workload(name)
    pool = K + W
    grads = park_gradients(torch, wl, pool)
    f = Flat(S, torch, wl, grads, K, W)
    gk_ms, _, _ = f.timed(S.sparsify_gaussiank)
    gk_stage, gk_nnz, gk_rounds = f.traced(S.sparsify_gaussiank)
    tk_ms, _, _ = f.timed(S.sparsify_topk)
    tk_stage, _, _ = f.traced(S.sparsify_topk)
    dom, nbytes, dom_gbps = dominant(gk_stage, wl.d)
    gk_bpe = gk_bytes_per_elem(gk_stage.listed, False)
    g = gbps(GK_BYTES_PER_ELEM, wl.d, float(np.mean(gk_nnz)), gk_ms)        # algorithmic bytes
    g_moved = gbps(gk_bpe, wl.d, float(np.mean(gk_nnz)), gk_ms)             # bytes as run
    tk_bpe = topk_bytes_per_elem(tk_stage.listed, False)
    t = gbps(tk_bpe, wl.d, float(wl.k), tk_ms)
    out = {"workload": wl.describe(), "gradient_pool": pool, "steps": K, "warmup": W,
           "working_set_MB": round(12 * wl.d / 1e6, 1),
           "gaussiank": {"ms_per_step": round(gk_ms, 5), "GBps": round(g, 2),
                         "pct_hbm_peak": round(100.0 * g / HBM_PEAK_GBPS, 2),
                         "bytes_per_elem": GK_BYTES_PER_ELEM, "steps_from_short_lists": gk_stage.listed,
                         "bytes_per_elem_moved": gk_bpe, "GBps_moved": round(g_moved, 2),
                         "pct_hbm_peak_moved": round(100.0 * g_moved / HBM_PEAK_GBPS, 2),
                         "nnz_mean": float(np.mean(gk_nnz)), "rounds_mean": float(np.mean(gk_rounds)),
                         "kernel_ms": {n: round(v, 5) for n, v in gk_stage.items()},
                         "kernel_ms_median": {n: round(v, 5) for n, v in gk_stage.median.items()}},
           "topk": {"ms_per_step": round(tk_ms, 5), "GBps": round(t, 2),
                    "pct_hbm_peak": round(100.0 * t / HBM_PEAK_GBPS, 2),
                    "bytes_per_elem": tk_bpe, "steps_from_short_lists": tk_stage.listed,
                    "kernel_ms": {n: round(v, 5) for n, v in tk_stage.items()},
                    "kernel_ms_median": {n: round(v, 5) for n, v in tk_stage.median.items()}},
           "roofline": {"bound": "hbm", "kernel": dom, "achieved": round(dom_gbps, 2),
                        "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                        "frac": round(dom_gbps / HBM_PEAK_GBPS, 4),
                        "bytes_per_launch": nbytes, "avg_ms": round(gk_stage[dom], 5)}}
    del f, grads
    torch.cuda.empty_cache()
    return out


def scatter_add_bench(S, torch, wl, grads, K, W):
    """Aggregation of P = 16 workers' Gaussian_k lists of this workload (each worker compresses
    its own gradient with a zero residual), scale 1/P: ms per call and algorithmic GB/s
    (4 bytes per element written + 8 bytes per pair read)."""
    import numpy as np
    P, d, k = 16, wl.d, wl.k
    cap = max(4 * k, 1024)
    b = S.Buffers.allocate(d, cap, 1, False, "cuda:0")
    idx = torch.zeros((P, cap), dtype=torch.int32, device="cuda:0")
    val = torch.zeros((P, cap), dtype=torch.float32, device="cuda:0")
    rec = torch.zeros((P, S.RESULT_BYTES), dtype=torch.uint8, device="cuda:0")
    for p in range(P):
        b.residual.zero_()
        S.sparsify_gaussiank(d, k, grads[p % len(grads)], b.residual, b.acc, idx[p], val[p], cap,
                             rec[p], b.workspace, b.workspace_nbytes)
    dense = torch.empty(d, dtype=torch.float32, device="cuda:0")
    status = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    stream = torch.cuda.current_stream()

    def call():
        S.sparsify_scatter_add(d, P, idx, val, cap, rec, dense, status, scale=1.0 / P,
                               nnz_stride_bytes=S.RESULT_BYTES, stream=stream)
    for _ in range(W):
        call()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(K):
        call()
    e1.record(stream)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / K
    pairs = int(S.decode_results(rec.reshape(-1))["nnz"].sum())
    nbytes = 4 * d + 8 * pairs
    g = nbytes / (ms * 1e-3) / 1e9
    return {"lists": P, "pairs": pairs, "scale": "1/16", "ms_per_call": round(ms, 5),
            "bytes_per_call": nbytes, "GBps": round(g, 2), "status": int(status.cpu()[0]),
            "roofline": {"bound": "hbm", "kernel": "scatter_add", "achieved": round(g, 2),
                         "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(g / HBM_PEAK_GBPS, 4)},
            "note": "4 B per element written + 8 B per pair read"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg3_resnet50")
    ap.add_argument("--inplace", action="store_true", help="acc aliases residual")
    ap.add_argument("--short-list", type=int, default=0,
                    help="-1: Top_k never builds the short lists in its accumulate pass")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip everything reported under `also` (other workloads, in place, layer-wise, "
                         "DGC_k, scatter-add) and the repeats")
    ap.add_argument("--tile-chunks", type=int, default=0, help="tuning: 4096-element chunks per workgroup")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain copy kernel of 4d bytes each way (counter scaling)")
    ap.add_argument("--scatter-add-only", action="store_true",
                    help="time only the aggregation of 16 workers' lists of the workload (for profiles)")
    ap.add_argument("--gradient-pool", type=int, default=0,
                    help="distinct gradients kept in HBM and cycled (default: one per step)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_1911_08772_amd import sparsify as S
    from paper_1911_08772_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3
    dev = "cuda:0"
    wl = synth.workload(args.workload)
    d, k = wl.d, wl.k
    K, W = args.steps, args.warmup
    n_grads = args.gradient_pool if args.gradient_pool > 0 else K + W

    if args.scatter_add_only:
        grads = park_gradients(torch, wl, 16)
        print(json.dumps({"workload": wl.describe(),
                          "scatter_add": scatter_add_bench(S, torch, wl, grads, K, W)}), flush=True)
        return 0
    grads = park_gradients(torch, wl, n_grads)   # before any timing
    f = Flat(S, torch, wl, grads, K, W, args.inplace, args.tile_chunks, args.short_list)
    cap, stream = f.cap, f.stream

    if args.calibration_copy:
        n4 = d - d % 4
        for _ in range(3):
            S.sparsify_calibration_copy(f.b.acc, grads[0], n4, stream=stream)
        torch.cuda.synchronize()

    gk_ms, gk_wall, gk_ev = f.timed(S.sparsify_gaussiank)
    gk_stage, gk_nnz, gk_rounds = f.traced(S.sparsify_gaussiank)
    tk_ms, tk_wall, tk_ev = f.timed(S.sparsify_topk)
    tk_stage, tk_nnz, _ = f.traced(S.sparsify_topk)
    gk_spread = tk_spread = None
    if not args.no_extras:
        gk_spread = f.spread(S.sparsify_gaussiank, 5)
        tk_spread = f.spread(S.sparsify_topk, 5)
    dg = None
    if not args.inplace and not args.no_extras:  # the sampling comparator of Sec. 4.3 (1 % sample)
        dg_ms, _, _ = f.timed(S.sparsify_dgck)
        dg_stage, dg_nnz, dg_rounds = f.traced(S.sparsify_dgck)
        dg = {"ms_per_step": round(dg_ms, 5), "nnz_mean": float(np.mean(dg_nnz)),
              "selections_mean": float(np.mean(dg_rounds)),
              "steps_from_short_lists": dg_stage.listed,
              "kernel_ms": {n: round(v, 5) for n, v in dg_stage.items()}}

    extras = {}
    if not args.no_extras:
        # the same chain with acc aliased to the residual (20 B per element)
        fi = Flat(S, torch, wl, grads, K, W, True)
        extras["inplace"] = {"gaussiank_ms": round(fi.timed(S.sparsify_gaussiank)[1], 5),
                             "topk_ms": round(fi.timed(S.sparsify_topk)[1], 5),
                             "note": "acc == residual: 16 B per element for Gaussian_k and 12 for Top_k when their short lists serve (20 and 28 otherwise)"}
        del fi
        # layer-wise call: 54 segments of the same total length, one launch sequence per step
        if wl.d == 25_557_032:
            seg = synth.workload("cfg4_segmented")
            caps = np.maximum(4 * seg.seg_k, 1024)
            out_off = np.concatenate([[0], np.cumsum(caps)]).astype(np.int64)
            L, ocap = int(seg.seg_k.size), int(out_off[-1])
            bs = S.Buffers.allocate(d, ocap, L, False, dev)
            d_off = torch.from_numpy(seg.seg_off).to(dev)
            d_k = torch.from_numpy(seg.seg_k).to(dev)
            d_oo = torch.from_numpy(out_off).to(dev)

            def timed_seg(mode):
                bs.residual.zero_()
                for s in range(W + K):
                    if s == W:
                        torch.cuda.synchronize()
                        t0 = time.perf_counter()
                    S.sparsify_segmented(L, d, d_off, d_k, mode, grads[s % n_grads], bs.residual, bs.acc,
                                         bs.out_idx, bs.out_val, d_oo, ocap, bs.result, bs.workspace,
                                         bs.workspace_nbytes, stream=stream)
                torch.cuda.synchronize()
                return (time.perf_counter() - t0) * 1e3 / K
            extras["segmented_54"] = {"gaussiank_ms": round(timed_seg(1), 5),
                                      "topk_ms": round(timed_seg(0), 5),
                                      "note": "cfg4 layout (54 segments) on the same gradients"}
            del bs
        extras["scatter_add"] = scatter_add_bench(S, torch, wl, grads, K, W)

    # `value`: the method's algorithmic bytes (accumulate 12, one count pass 4, compaction 8: the
    # 24 B per element the target is stated in, 20 with acc == residual) over the time; what the
    # kernels as run move (20 B with the short lists) is given beside it
    gk_alg_bpe = GK_INPLACE_BYTES_PER_ELEM if args.inplace else GK_BYTES_PER_ELEM
    gk_bpe = gk_bytes_per_elem(gk_stage.listed, args.inplace)
    tk_bpe = topk_bytes_per_elem(tk_stage.listed, args.inplace)
    gk_gbps = gbps(gk_alg_bpe, d, float(np.mean(gk_nnz)), gk_ms)
    gk_moved_gbps = gbps(gk_bpe, d, float(np.mean(gk_nnz)), gk_ms)
    tk_gbps = gbps(tk_bpe, d, float(k), tk_ms)
    dom, dom_bytes, dom_gbps = dominant(gk_stage, d, args.inplace)
    traffic, traffic_source = read_traffic(args.workload, dom)

    if not args.no_extras and args.workload == "cfg3_resnet50":
        # the workloads beside the headline: beyond the last-level cache, and below the headline size
        del f, grads
        torch.cuda.empty_cache()
        for name in ("cfg5_lstm", "cfg2_vgg16"):
            extras[name] = side_workload(S, torch, synth, name, K, W)

    out = {
        "metric": (f"Gaussian-k sparsify GB/s (algorithmic bytes: {gk_alg_bpe} B per element) at d=25.6M, rho=0.001; exact Top-k beside it"
                   if args.workload == "cfg3_resnet50" else
                   f"Gaussian-k sparsify GB/s (algorithmic bytes: {gk_alg_bpe} B per element) on {wl.name}; exact Top-k beside it"),
        "value": round(gk_gbps, 2), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(gk_ms, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.describe() + ", residual carried",
                   "acc": "in-place" if args.inplace else "separate", "cap": cap,
                   "gradient_pool": n_grads},
        "elements_per_s": round(d / (gk_ms * 1e-3), 1),
        "pct_hbm_peak": round(100.0 * gk_gbps / HBM_PEAK_GBPS, 2),   # of algorithmic bytes, as `value`
        # the kernels as run move fewer bytes than the method's count when the short lists serve
        "GBps_moved": round(gk_moved_gbps, 2),
        "pct_hbm_peak_moved": round(100.0 * gk_moved_gbps / HBM_PEAK_GBPS, 2),
        "gaussiank": {"ms_per_step": round(gk_ms, 5), "wall_ms": round(gk_wall, 5),
                      "event_ms": round(gk_ev, 5), "bytes_per_elem": gk_alg_bpe,
                      "steps_from_short_lists": gk_stage.listed,
                      # what the kernels as run move (with the short lists the compaction does
                      # not stream the vector again) and the rate on those bytes
                      "bytes_per_elem_moved": gk_bpe, "GBps_moved": round(gk_moved_gbps, 2),
                      "pct_hbm_peak_moved": round(100.0 * gk_moved_gbps / HBM_PEAK_GBPS, 2),
                      "nnz_mean": float(np.mean(gk_nnz)), "rounds_mean": float(np.mean(gk_rounds)),
                      "spread": gk_spread,
                      "kernel_ms": {n: round(v, 5) for n, v in gk_stage.items()},
                         "kernel_ms_median": {n: round(v, 5) for n, v in gk_stage.median.items()}},
        "topk": {"ms_per_step": round(tk_ms, 5), "GBps": round(tk_gbps, 2),
                 "elements_per_s": round(d / (tk_ms * 1e-3), 1),
                 "pct_hbm_peak": round(100.0 * tk_gbps / HBM_PEAK_GBPS, 2),
                 "bytes_per_elem": tk_bpe, "steps_from_short_lists": tk_stage.listed,
                 "spread": tk_spread,
                 # context only (Sec. 3.3: a tensor library's topk() on a Tesla V100, same d and k)
                 "paper_v100_ms": 400.0 if (wl.d == 25_557_032 and k == 25_558) else None,
                 "kernel_ms": {n: round(v, 5) for n, v in tk_stage.items()},
                    "kernel_ms_median": {n: round(v, 5) for n, v in tk_stage.median.items()}},
        "gaussiank_speedup_over_topk": round(tk_ms / gk_ms, 3),
        "dgck": dg,
        "also": extras,
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": round(dom_gbps, 2),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(dom_gbps / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "traffic_source": traffic_source,
                     "bytes_per_launch": dom_bytes, "avg_ms": round(gk_stage[dom], 5)},
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, cap)
    print(json.dumps(out), flush=True)
    return 0


def kernel_sources_digest() -> str:
    """Short SHA-256 over the kernel sources (file names and contents, in name order): the
    committed profile summaries carry the digest of the sources they were measured on."""
    import hashlib
    csrc = os.path.join(ROOT, "paper_1911_08772_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".h", ".hip", ".c")):
            h.update(name.encode())
            with open(os.path.join(csrc, name), "rb") as fh:
                h.update(fh.read())
    return h.hexdigest()[:16]


def read_traffic(workload: str, kernel: str):
    """HBM-side bytes per launch of `kernel` from the committed rocprofv3 --pmc summary of this
    workload (FETCH_SIZE and WRITE_SIZE scaled by a plain copy kernel) and where the figure comes
    from: it is a profile of the committed kernels, not a counter read during this run (the
    summary names the digest of the kernel sources it was measured on; a figure measured on
    other sources is still returned, and said to be).  None when there is no summary."""
    rel = os.path.join("profiles", f"bench_{workload}_hbm_traffic.txt")
    path = os.path.join(ROOT, rel)
    try:
        lines = open(path).read().splitlines()
        same = f"kernel sources digest={kernel_sources_digest()}" in lines
        for line in lines:
            if line.startswith(f"traffic kernel={kernel} "):
                value = float(line.split("bytes_per_launch=")[1])
                if not same:
                    return value, f"{rel} (committed rocprofv3 --pmc summary; measured on other kernel sources than these)"
                return value, f"{rel} (committed rocprofv3 --pmc summary, not measured in this run)"
    except (OSError, ValueError):
        pass
    return None, None


def cpu_baseline(wl, cap):
    """The CPU oracle as it stands, single thread, on a bounded sample of the same workload:
    the first error-feedback steps of the chain (accumulate + Gaussian_k), about 10-20 s."""
    import numpy as np

    from oracle import oracle as O
    d, k = wl.d, wl.k
    g = np.empty(d, np.float32)
    acc = np.empty(d, np.float32)
    eps = np.zeros(d, np.float32)
    nxt = np.zeros(d, np.float32)
    idx, val = np.empty(cap, np.uint32), np.empty(cap, np.float32)
    wl.grad(0, out=g)
    O.accumulate(g, eps, out=acc)           # touch every page once before timing
    O.gaussiank(acc, k, cap=cap, eps_out=nxt, idx=idx, val=val)
    eps[:] = 0
    pool = [wl.grad(s) for s in range(8)]   # fresh gradients, cycled
    spent, steps, nnz = 0.0, 0, []
    budget_s, max_steps = 12.0, 1000
    while spent < budget_s and steps < max_steps:
        g = pool[steps % len(pool)]
        t0 = time.perf_counter()
        O.accumulate(g, eps, out=acc)
        _, _, _, r = O.gaussiank(acc, k, cap=cap, eps_out=nxt, idx=idx, val=val)
        spent += time.perf_counter() - t0
        eps, nxt = nxt, eps
        nnz.append(r.nnz)
        steps += 1
    ms = spent / steps * 1e3
    t0 = time.perf_counter()
    O.topk(acc, k, eps_out=nxt, idx=idx, val=val)
    topk_ms = (time.perf_counter() - t0) * 1e3
    return {"value": round((GK_BYTES_PER_ELEM * d + 8.0 * float(np.mean(nnz))) / (ms * 1e-3) / 1e9, 4),
            "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"{steps} error-feedback steps of {wl.name} (accumulate + Gaussian_k, 8 gradients "
                      f"cycled), single thread, {spent:.1f} s",
            "ms_per_step": round(ms, 2), "topk_ms_one_step": round(topk_ms, 2)}


if __name__ == "__main__":
    sys.exit(main())

"""Operator time of Gaussian_k, exact Top_k and DGC_k (1 % sample) against the vector length d (k = 0.001 d),
the shape of the paper's GPU-efficiency experiment (Sec. 4.3: d from 1 M to 512 M on one GPU).

For each d: seeded N(0, 1e-3) gradients resident in HBM, residual carried over the steps,
median time of one call over the timed steps.  Prints one JSON line per d and a final table.
Not the headline benchmark (that is bench.py); same kernels, second workload.
"""
import argparse
import json
import os
import statistics
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

DEFAULT_SIZES = [1 << 20, 1 << 22, 1 << 24, 20_000_000, 1 << 26, 100_000_000, 1 << 28,
                 400_000_000, 1 << 29]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--sizes", type=int, nargs="*", default=DEFAULT_SIZES)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--pool", type=int, default=4, help="distinct gradients cycled through")
    ap.add_argument("--tile-chunks", type=int, default=0, help="tuning: 4096-element chunks per workgroup")
    args = ap.parse_args()

    import numpy as np
    import torch

    from paper_1911_08772_amd import sparsify as S
    from paper_1911_08772_amd import synth

    if not torch.cuda.is_available():
        print("bench_sweep.py: no GPU visible", file=sys.stderr)
        return 3
    dev = "cuda:0"
    rows = []
    for d in args.sizes:
        k = synth.k_of(d, 1000)
        cap = max(4 * k, 1024)
        host = np.empty(d, np.float32)
        grads = []
        for s in range(args.pool):
            synth.normal(d, synth.BASE_SEED + 9, s, 1e-3, out=host)
            g = torch.empty(d, dtype=torch.float32, device=dev)
            g.copy_(torch.from_numpy(host))
            grads.append(g)
        b = S.Buffers.allocate(d, cap, 1, False, dev)
        stream = torch.cuda.current_stream()
        out = {"d": d, "k": k}
        # bytes per element of the passes as run: (three passes over the vector, with short lists)
        for name, fn, bpes in (("gaussiank", S.sparsify_gaussiank, (24, 20)), ("topk", S.sparsify_topk, (24, 16)),
                               ("dgck", S.sparsify_dgck, (24, 16))):
            b.residual.zero_()
            times = []
            for s in range(args.warmup + args.steps):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                fn(d, k, grads[s % args.pool], b.residual, b.acc, b.out_idx, b.out_val, cap, b.result,
                   b.workspace, b.workspace_nbytes, stream=stream, tile_chunks=args.tile_chunks)
                e1.record(stream)
                torch.cuda.synchronize()
                if s >= args.warmup:
                    times.append(e0.elapsed_time(e1))
            ms = statistics.median(times)
            res = S.decode_results(b.result)[0]
            bpe = bpes[1] if int(res["flags"]) & S.F_SHORTLIST else bpes[0]   # (the last step's way)
            out[name] = {"ms": round(ms, 5), "bytes_per_elem": bpe,
                         "GBps": round(bpe * d / (ms * 1e-3) / 1e9, 1),
                         "Gelem_per_s": round(d / (ms * 1e-3) / 1e9, 2), "nnz_last": int(res["nnz"])}
        out["topk_over_gaussiank"] = round(out["topk"]["ms"] / out["gaussiank"]["ms"], 3)
        out["dgck_over_gaussiank"] = round(out["dgck"]["ms"] / out["gaussiank"]["ms"], 3)
        print(json.dumps(out), flush=True)
        rows.append(out)
        del grads, b
        torch.cuda.empty_cache()
    print(f"{'d':>12} {'k':>8} {'gaussiank ms':>13} {'GB/s':>8} {'topk ms':>9} {'GB/s':>8} {'ratio':>6} "
          f"{'dgck ms':>9} {'ratio':>6}")
    for r in rows:
        print(f"{r['d']:>12} {r['k']:>8} {r['gaussiank']['ms']:>13.4f} {r['gaussiank']['GBps']:>8.0f} "
              f"{r['topk']['ms']:>9.4f} {r['topk']['GBps']:>8.0f} {r['topk_over_gaussiank']:>6.2f} "
              f"{r['dgck']['ms']:>9.4f} {r['dgck_over_gaussiank']:>6.2f}")
    return 0


if __name__ == "__main__":
    sys.exit(main())

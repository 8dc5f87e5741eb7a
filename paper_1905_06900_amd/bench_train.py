"""Throughput of encoding and of the training steps (Sec. 3.2, Alg. 2) on one MI355X, at the shapes of the
SIFT-like workload (PQ 8x16: m = 8, dsub = 16, 2^16 centroids per sub-quantizer, derived codebooks of 2^8).

One JSON line per measurement; the matrix-core figure of the assignment kernel counts 2 n 2^16 D flop
against the chip's double-precision matrix peak.

    python -m paper_1905_06900_amd.bench_train [--n 1000000]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

from paper_1905_06900_amd import binding, synth  # noqa: E402

FP64_MFMA_PEAK_TFLOPS = 78.6


def timed(fn, reps=3):
    fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / reps


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=1_000_000, help="vectors to encode / training points")
    args = ap.parse_args()
    assert torch.cuda.is_available(), "bench_train needs a GPU"
    dev = "cuda:0"
    w = synth.WORKLOADS[1]
    m, dsub, b, bbar, n = w.m, w.dsub, 16, 8, args.n
    cb = synth.hierarchical_codebooks(m, dsub, b, w.pbits, synth._uniform(0.0, 160.0, dev), 12.0, dev, w.seed + 1)
    x = synth.sift_like(n, dev, w.seed + 2, w.seed + 3)

    s = timed(lambda: binding.encode(x, cb), reps=2)
    flop = 2.0 * n * (1 << b) * m * dsub
    print(json.dumps({"what": "encode", "shape": "PQ %dx%d, dsub %d" % (m, b, dsub), "vectors": n, "seconds": round(s, 4),
                      "vectors_per_s": round(n / s, 1), "seconds_per_million": round(s * 1e6 / n, 3),
                      "mfma_tflops": round(flop / s / 1e12, 2), "frac_of_fp64_mfma_peak": round(flop / s / 1e12 / FP64_MFMA_PEAK_TFLOPS, 4)}))

    pts = x[:, :dsub].contiguous()
    init = pts[: 1 << b].clone()
    s1 = timed(lambda: binding.kmeans(pts, init, 1), reps=2)
    s0 = timed(lambda: binding.kmeans(pts, init, 0), reps=2)
    print(json.dumps({"what": "kmeans iteration (assign + means)", "points": n, "d": dsub, "k": 1 << b,
                      "seconds_per_iteration": round(s1 - s0, 4), "assign_only_seconds": round(s0, 4)}))

    temp = cb[0].contiguous()
    sinit = temp[: 1 << bbar].clone()
    s = timed(lambda: binding.kmeans_same_size(temp, sinit, 1), reps=2)
    print(json.dumps({"what": "same-size k-means iteration", "points": 1 << b, "groups": 1 << bbar, "d": dsub,
                      "seconds_per_iteration": round(s, 4)}))

    nt = min(n, 262144)
    init_cb = torch.stack([x[: 1 << b, j * dsub:(j + 1) * dsub] for j in range(m)]).contiguous()
    t0 = time.perf_counter()
    binding.build_quantizers(x[:nt].contiguous(), init_cb, bbar, 4, 2)
    torch.cuda.synchronize()
    print(json.dumps({"what": "build_quantizers (Alg. 2, 4 k-means + 2 same-size iterations per sub-quantizer)", "train_points": nt,
                      "m": m, "seconds": round(time.perf_counter() - t0, 3)}))
    return 0


if __name__ == "__main__":
    sys.exit(main())

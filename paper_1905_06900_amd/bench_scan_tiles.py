"""Pass-one scan over the headline code array for a sweep of batch sizes and query tiles.

The single-pass scan keeps the tables of a tile of 16, 32 or 64 queries in LDS and streams the codes
once per tile, so the tile trades LDS lookups per byte of code stream against passes over the stream.
For every (queries, tile, r) this prints one JSON line with the time of the scan kernel (and, beside it, of
the sample histogram and of the final selection), the
(query, code) pairs per second, and the code stream rate = passes x N x bytes per code / time, which
is what the kernel loads (from HBM, or from the L2 when several tiles walk the same codes together).

    python -m paper_1905_06900_amd.bench_scan_tiles [--n 100000000] [--queries 16,64,1024] [--r 10,4000]
"""
from __future__ import annotations

import argparse
import json
import os
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

from paper_1905_06900_amd import binding, synth  # noqa: E402

HBM_PEAK_GBS = 8000.0
TILES = {16: binding.SCAN_TILE16, 32: binding.SCAN_TILE32, 64: binding.SCAN_TILE64}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=None, help="codes (default: the headline workload's 100M)")
    ap.add_argument("--queries", default="16,32,64,256,1024")
    ap.add_argument("--r", default="10,4000")
    ap.add_argument("--reps", type=int, default=3)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        print("bench_scan_tiles.py needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    dev = "cuda:0"
    qs = [int(x) for x in args.queries.split(",")]
    rs = [int(x) for x in args.r.split(",")]
    w = synth.WORKLOADS[2]
    w = synth.scaled(w, N=args.n or w.N, Q=max(qs))
    data = synth.make_flat(w, dev)
    cb, codes, queries = data["codebooks"], data["codes"], data["queries"]
    derived = binding.derive_codebooks(cb)
    code_bytes = 2 * w.m
    for r in rs:
        for nq in qs:
            qtab, _, _ = binding.build_small_tables(queries[:nq].contiguous(), derived, codes, r)
            ws = torch.empty(binding.scan_workspace_bytes(w.N, w.m, nq, r), dtype=torch.uint8, device=dev)
            for tile, mode in TILES.items():
                for _ in range(2):
                    binding.scan_candidates(codes, qtab, r, workspace=ws, mode=mode)
                torch.cuda.synchronize()
                binding.profile_enable(True)
                for _ in range(args.reps):
                    binding.scan_candidates(codes, qtab, r, workspace=ws, mode=mode)
                torch.cuda.synchronize()
                st = binding.profile_read()
                binding.profile_enable(False)
                ms = st["scan_fast"][0] / args.reps
                other = {k: round(st[k][0] / args.reps, 4) for k in ("scan_hist", "select") if k in st}
                passes = -(-nq // tile)
                stream = passes * w.N * code_bytes / (ms * 1e-3) / 1e9
                print(json.dumps({
                    "workload": w.name, "N": w.N, "queries": nq, "r": r, "query_tile": tile, "passes": passes,
                    "scan_ms": round(ms, 4), "pairs_per_s": round(w.N * nq / (ms * 1e-3), 1),
                    "code_stream_GBs": round(stream, 1), "frac_of_hbm_peak": round(stream / HBM_PEAK_GBS, 4),
                    "queries_per_s_scan_only": round(nq / (ms * 1e-3), 1), "sample_and_redo_ms": other.get("scan_hist"),
                    "select_ms": other.get("select"),
                }), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())

"""End-to-end queries/s of all five workloads (the four flat ones and the inverted-index one).

One JSON line per workload: the whole search (tables, scan, selection, refine, top-k; for the
inverted index also the coarse probe) over the full batch at full size, inputs resident on the
device, derived codebooks excluded as index build.  `bench.py` is the headline measurement; this
script only puts the other workloads beside it.

    python -m paper_1905_06900_amd.bench_configs [--cfgs 0,1,2,3,4] [--steps 3]
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


def time_steps(step, steps: int, warmup: int = 1):
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    binding.profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    stages = binding.profile_read()
    binding.profile_enable(False)
    return elapsed / steps, {s: round(v[0] / steps, 3) for s, v in stages.items() if v[1]}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--cfgs", default="0,1,2,3,4")
    ap.add_argument("--steps", type=int, default=3)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        print("bench_configs.py needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    dev = "cuda:0"
    for c in (int(x) for x in args.cfgs.split(",")):
        w = synth.WORKLOADS[c]
        if w.kind == "flat":
            d = synth.make_flat(w, dev)
            cb, codes, queries = d["codebooks"], d["codes"], d["queries"]
            derived = binding.derive_codebooks(cb)
            ws = torch.empty(binding.search_workspace_bytes(w.N, w.m, w.Q, w.r, 0), dtype=torch.uint8, device=dev)
            ids = torch.empty((w.Q, w.k), dtype=torch.uint32, device=dev)
            dist = torch.empty((w.Q, w.k), dtype=torch.float32, device=dev)

            def step():
                binding.search(queries, cb, derived, codes, w.r, w.k, 0, ws, ids, dist)
        else:
            d = synth.make_ivf(w, dev)
            cb, coarse, offsets = d["codebooks"], d["coarse"], d["offsets"]
            codes, queries = d["codes"], d["queries"]
            derived = binding.derive_codebooks(cb)
            plane = binding.pack_low_bytes(codes)                # index build: the bytes pass one reads

            def step():
                probe = binding.ivf_probe(queries, coarse, w.nprobe)
                qtab, _ = binding.ivf_build_small_tables(queries, coarse, probe, derived, codes, offsets, w.r)
                cand_id, _, _ = binding.ivf_scan_candidates(plane, offsets, probe, qtab, w.r)
                binding.ivf_refine_topk(queries, coarse, cb, codes, offsets, probe, cand_id, w.k)
        sec, stages = time_steps(step, args.steps)
        print(json.dumps({
            "workload": w.name, "kind": w.kind, "N": w.N, "queries": w.Q, "m": w.m, "dsub": w.dsub, "r": w.r,
            "k": w.k, "queries_per_s": round(w.Q / sec, 1), "ms_per_step": round(sec * 1e3, 3),
            "stage_ms_per_step": stages,
        }), flush=True)
        del d, codes, queries, cb
        torch.cuda.empty_cache()
    return 0


if __name__ == "__main__":
    sys.exit(main())

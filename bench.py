#!/usr/bin/env python3
"""Benchmark of the two-pass derived-codebook PQ search on one MI355X.

One step = the whole hot path (small tables + quantizer, scan + candidate selection, full tables,
refine + top-k) for one batch of queries over the resident code array, through the C ABI.
Prints ONE JSON line.  Workload: BASELINE's headline configuration (flat PQ 8x16, N = 100M,
4096 queries, r = 4000, k = 100) unless --cfg / --n / --q say otherwise.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
SCAN_STAGES = ("scan_fast", "scan_hist", "scan_tiecount", "scan_collect")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--cfg", type=int, default=2, help="workload index in BASELINE.json (flat ones)")
    ap.add_argument("--n", type=int, default=None, help="override database size (experiments only)")
    ap.add_argument("--q", type=int, default=None, help="override query batch (experiments only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--chunk", type=int, default=0, help="queries per chunk of the fused search (0 = default)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also launch one 1 GiB calibration_copy_kernel (for scaling rocprofv3 --pmc traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_1905_06900_amd import binding, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    binding.lib()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = synth.WORKLOADS[args.cfg]
    assert w.kind == "flat", "bench.py times the flat path; the IVF variant has its own tests"
    w = synth.scaled(w, N=args.n, Q=args.q)

    t0 = time.perf_counter()
    data = synth.make_flat(w, dev)
    cb, codes, queries = data["codebooks"], data["codes"], data["queries"]
    derived = binding.derive_codebooks(cb)                       # index build, not timed
    ws = torch.empty(binding.search_workspace_bytes(w.N, w.m, w.Q, w.r, args.chunk), dtype=torch.uint8, device=dev)
    ids = torch.empty((w.Q, w.k), dtype=torch.uint32, device=dev)
    dist = torch.empty((w.Q, w.k), dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    setup_s = time.perf_counter() - t0

    def step():
        binding.search(queries, cb, derived, codes, w.r, w.k, args.chunk, ws, ids, dist)

    if args.calibration_copy:
        a = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        b = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        a.zero_()
        binding.profile_copy(a, b)
        torch.cuda.synchronize()
        del a, b
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    binding.profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    stages = binding.profile_read()
    binding.profile_enable(False)

    ms_per_step = elapsed / args.steps * 1e3
    qps = w.Q * args.steps / elapsed

    # Roofline of the dominant kernel (the scan over the code stream).
    code_bytes = 2 * w.m                                         # bytes per code per pass, as stored
    qt = binding.scan_query_tile(w.m)
    dom = max(SCAN_STAGES, key=lambda s: stages.get(s, (0.0, 0))[0])
    dom_ms, dom_launches = stages[dom]
    passes_per_step = sum((min(binding.search_chunk(w.m, w.Q, args.chunk), w.Q - q0) + qt - 1) // qt
                          for q0 in range(0, w.Q, binding.search_chunk(w.m, w.Q, args.chunk)))
    launches_per_step = dom_launches / args.steps
    chunk = binding.search_chunk(w.m, w.Q, args.chunk)
    bytes_per_launch = passes_per_step * w.N * code_bytes / launches_per_step
    avg_launch_s = dom_ms / dom_launches * 1e-3
    achieved = bytes_per_launch / avg_launch_s / 1e9
    scan_ms = sum(stages.get(s, (0.0, 0))[0] for s in SCAN_STAGES) / args.steps
    # HBM-side bytes per launch of that kernel from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    # WRITE_SIZE scaled by the calibration copy); only meaningful for the workload it was taken on.
    traffic = None
    prof = os.path.join(ROOT, "profiles", "scan_fast_cfg2_counters.txt")
    if dom == "scan_fast" and args.cfg == 2 and args.n is None and args.q is None and args.chunk == 0 and os.path.exists(prof):
        import re
        mt = re.search(r"measured traffic below the L2 = .*?\((\d+) bytes\)", open(prof).read())
        if mt:
            traffic = int(mt.group(1))
    roofline = {
        "bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
        "bytes_per_launch": bytes_per_launch, "avg_launch_ms": round(dom_ms / dom_launches, 4),
        "launches_per_step": launches_per_step, "queries_per_pass": qt,
        "code_passes_per_step": passes_per_step, "codes_per_pass": w.N,
        "pairs_per_s": round(w.N * w.Q / (scan_ms * 1e-3), 1) if scan_ms > 0 else None,
    }

    # The same scan with the 16-query tile on one chunk: a quarter of the lookups per byte of code stream,
    # i.e. the configuration in which pass one is bound by the stream and not by LDS lookups.  Context for
    # `roofline` (which describes the configuration that gives the most queries/s), not part of `value`.
    stream_variant = None
    if w.m == 8 and dom == "scan_fast":
        nq_v = min(chunk, w.Q)
        qtab_v, _, _ = binding.build_small_tables(queries[:nq_v].contiguous(), derived, codes, w.r)
        ws_v = torch.empty(binding.scan_workspace_bytes(w.N, w.m, nq_v, w.r), dtype=torch.uint8, device=dev)
        binding.scan_candidates(codes, qtab_v, w.r, workspace=ws_v, mode=binding.SCAN_TILE16)
        torch.cuda.synchronize()
        binding.profile_enable(True)
        for _ in range(2):
            binding.scan_candidates(codes, qtab_v, w.r, workspace=ws_v, mode=binding.SCAN_TILE16)
        torch.cuda.synchronize()
        st_v = binding.profile_read()
        binding.profile_enable(False)
        plan_v = binding.scan_plan(w.N, w.m, nq_v, w.r, binding.SCAN_TILE16)
        ms_v = st_v["scan_fast"][0] / st_v["scan_fast"][1]
        bytes_v = plan_v["tiles"] * w.N * code_bytes
        stream_variant = {
            "query_tile": 16, "queries": nq_v, "bound": "hbm", "achieved": round(bytes_v / (ms_v * 1e-3) / 1e9, 1),
            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(bytes_v / (ms_v * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "avg_launch_ms": round(ms_v, 4), "bytes_per_launch": bytes_v,
        }
        del ws_v, qtab_v

    out = {
        "metric": "queries/sec at k=100 + scan GB/s vs HBM peak (PQ 8x16, N=100M, 1 GPU)",
        "value": round(qps, 2), "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8 scan / f32 refine", "data": "synthetic",
        "config": {"workload": w.name, "N": w.N, "queries": w.Q, "m": w.m, "dsub": w.dsub, "r": w.r, "k": w.k,
                   "code_bytes": code_bytes, "seed": w.seed},
        "roofline": roofline,
        "scan_stream_variant": stream_variant,
        "stage_ms_per_step": {s: round(v[0] / args.steps, 3) for s, v in stages.items() if v[1]},
        "setup_s": round(setup_s, 2),
    }

    if not args.no_cpu_baseline:
        import oracle
        threads = oracle.num_threads()
        nsample = min(w.Q, 2 * threads)
        cb_np, codes_np = synth.to_numpy(cb), synth.to_numpy(codes)
        q_np = synth.to_numpy(queries)[:nsample]
        der_np = oracle.derive_codebooks(cb_np)
        t0 = time.perf_counter()
        ref = oracle.search_flat(cb_np, der_np, codes_np, q_np, w.r, w.k)
        cpu_s = time.perf_counter() - t0
        got = synth.to_numpy(ids)[:nsample]
        out["cpu_baseline"] = {
            "value": round(nsample / cpu_s, 3), "unit": "queries/s", "cores": threads, "kind": "oracle",
            "sample": "%d queries of the batch at full N=%d, one query per thread" % (nsample, w.N),
            "seconds": round(cpu_s, 2),
            "result_ids_equal_fraction": float((got == ref["ids"]).mean()),
        }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())

#!/usr/bin/env python3
"""Benchmark of the two-pass derived-codebook PQ search on one MI355X.

One step = the whole hot path for one batch of queries over the resident code array, through the C
ABI: small tables + quantizer, scan + candidate selection, full tables, refine + top-k (flat
workloads, one dcpq_search call) or coarse probe, residual tables, scan of the probed lists, residual
refine (inverted-index workload, one dcpq_ivf_search call).  Prints ONE JSON line.

The headline workload is BASELINE's flat PQ 8x16, N = 100M, 4096 queries, r = 4000, k = 100
(--cfg 2, the default).  Without --cfg the other four workloads are measured as well, more briefly,
and reported under "other_workloads" of the same line; a failure there is recorded, never raised.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
FP64_MFMA_PEAK_TFLOPS = 78.6   # MI355X published dense fp64 matrix rate
SCAN_STAGES = ("scan_fast", "scan_hist", "scan_tiecount", "scan_collect")
METRIC = "queries/sec at k=100 + scan GB/s vs HBM peak (PQ 8x16, N=100M, 1 GPU)"


def timed(step, steps, warmup, binding, torch):
    """W warm-up steps, then exactly K timed steps between synchronizations (-> elapsed); then the same K steps
    once more with the library's per-stage HIP events switched on (-> stage times: the events cost a few
    microseconds per kernel, which the timed steps should not carry)."""
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    binding.profile_enable(True)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    stages = binding.profile_read()
    binding.profile_enable(False)
    return elapsed, stages


def committed_traffic(kernel, workload):
    """HBM-side bytes per launch from the committed rocprofv3 --pmc summary of this kernel and workload
    (FETCH_SIZE + WRITE_SIZE scaled by the calibration copy), or None."""
    prof = os.path.join(ROOT, "profiles", "%s_%s_counters.txt" % (kernel, workload.split("_")[0]))
    if not os.path.exists(prof):
        return None
    m = re.search(r"measured traffic below the L2 = .*?\((\d+) bytes\)", open(prof).read())
    return int(m.group(1)) if m else None


def hbm_roofline(kernel, bytes_per_launch, total_ms, launches, steps, workload, limiter, extra=None):
    avg_ms = total_ms / launches
    achieved = bytes_per_launch / (avg_ms * 1e-3) / 1e9
    traffic = committed_traffic(kernel, workload)
    r = {"bound": "hbm", "kernel": kernel, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
         "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "bytes_per_launch": bytes_per_launch,
         "avg_launch_ms": round(avg_ms, 4), "launches_per_step": launches / steps, "limiter": limiter}
    if traffic is not None:
        r["hbm_traffic_frac"] = round(traffic / (avg_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    if extra:
        r.update(extra)
    return r


def calibration_copy(binding, torch, dev):
    """One launch of the library's 1 GiB copy kernel: its known traffic scales what rocprofv3 --pmc
    reports for FETCH_SIZE and WRITE_SIZE in the same run."""
    a = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    b = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    a.zero_()
    binding.profile_copy(a, b)
    torch.cuda.synchronize()
    del a, b


def run_flat(w, args, steps, warmup, with_cpu, headline):
    import torch
    from paper_1905_06900_amd import binding, synth
    dev = "cuda:0"
    t0 = time.perf_counter()
    data = synth.make_flat(w, dev)
    cb, codes, queries = data["codebooks"], data["codes"], data["queries"]
    derived = binding.derive_codebooks(cb)                       # index build, not timed
    ws = torch.empty(binding.search_workspace_bytes(w.N, w.m, w.Q, w.r, args.chunk), dtype=torch.uint8, device=dev)
    ids = torch.empty((w.Q, w.k), dtype=torch.uint32, device=dev)
    dist = torch.empty((w.Q, w.k), dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    setup_s = time.perf_counter() - t0

    refine_mode = {"auto": binding.REFINE_AUTO, "tables": binding.REFINE_TABLES, "direct": binding.REFINE_DIRECT,
                   "split": binding.REFINE_SPLIT}[args.refine]

    def step():
        binding.search(queries, cb, derived, codes, w.r, w.k, args.chunk, ws, ids, dist, refine_mode)

    if args.calibration_copy:
        calibration_copy(binding, torch, dev)
    elapsed, stages = timed(step, steps, warmup, binding, torch)
    ms_per_step = elapsed / steps * 1e3
    qps = w.Q * steps / elapsed

    # Roofline of the dominant kernel.
    code_bytes = 2 * w.m                                         # bytes per code per pass, as stored
    chunk = binding.search_chunk(w.m, w.Q, args.chunk)
    # the dominant kernel among those a roofline is defined for (the selection and the small tables are
    # several short launches each; on the smallest workload their launch latencies add up to more than the scan)
    dom = max((s for s in stages if s in SCAN_STAGES + ("full_tables", "refine_topk") and stages[s][1]),
              key=lambda s: stages[s][0])
    dom_ms, dom_launches = stages[dom]
    scan_ms = sum(stages.get(s, (0.0, 0))[0] for s in SCAN_STAGES) / steps
    if dom == "full_tables":
        # 2 Q 65536 D flop per step on the double-precision matrix cores, and 4 Q m 65536 bytes of
        # table writes: the bound is whichever roof the launch is closer to
        flops = 2.0 * w.Q * 65536 * w.D / (dom_launches / steps)
        wbytes = 4.0 * w.Q * w.m * 65536 / (dom_launches / steps)
        avg_s = dom_ms / dom_launches * 1e-3
        f_mfma, f_hbm = flops / avg_s / 1e12 / FP64_MFMA_PEAK_TFLOPS, wbytes / avg_s / 1e9 / HBM_PEAK_GBS
        if f_mfma >= f_hbm:
            roofline = {"bound": "mfma", "kernel": dom, "achieved": round(flops / avg_s / 1e12, 2),
                        "peak": FP64_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(f_mfma, 4),
                        "traffic": committed_traffic(dom, w.name), "flops_per_launch": flops,
                        "avg_launch_ms": round(avg_s * 1e3, 4), "launches_per_step": dom_launches / steps,
                        "limiter": "fp64 matrix instructions (K = dsub = %d per sub-quantizer)" % w.dsub}
        else:
            roofline = hbm_roofline(dom, wbytes, dom_ms, dom_launches, steps, w.name, "table writes to HBM")
    elif dom == "refine_topk":
        # pass two: per candidate one code and m centroid rows (on demand) or m table entries
        direct = binding.search_refine_mode(w.m, w.dsub, w.b, w.Q, w.r, refine_mode) != binding.REFINE_TABLES
        per_cand = code_bytes + w.m * (4 * w.dsub if direct else 4)
        roofline = hbm_roofline(dom, float(w.Q) * w.r * per_cand / (dom_launches / steps), dom_ms, dom_launches, steps, w.name,
                                "scattered reads (one code and m %s per candidate)" % ("centroid rows" if direct else "table entries"))
    else:
        qt = binding.scan_plan(w.N, w.m, min(chunk, w.Q), w.r)["query_tile"]
        passes_per_step = sum((min(chunk, w.Q - q0) + qt - 1) // qt for q0 in range(0, w.Q, chunk))
        launches_per_step = dom_launches / steps
        bytes_per_launch = passes_per_step * w.N * code_bytes / launches_per_step
        limiter = ("LDS row reads + the SIMDs' vector/matrix instruction port (%d queries share one pass over the "
                   "codes; the passes in flight share the stream through the L2)" % qt) if dom == "scan_fast" \
            else "LDS byte gathers (three-pass scan)"
        roofline = hbm_roofline(dom, bytes_per_launch, dom_ms, dom_launches, steps, w.name, limiter, {
            "queries_per_pass": qt, "code_passes_per_step": passes_per_step, "codes_per_pass": w.N,
            "pairs_per_s": round(w.N * w.Q / (scan_ms * 1e-3), 1) if scan_ms > 0 else None})

    out = {
        "value": round(qps, 2), "unit": "queries/s", "ms_per_step": round(ms_per_step, 3),
        "config": {"workload": w.name, "N": w.N, "queries": w.Q, "m": w.m, "dsub": w.dsub, "r": w.r, "k": w.k,
                   "code_bytes": code_bytes, "seed": w.seed},
        "roofline": roofline,
        "stage_ms_per_step": {s: round(v[0] / steps, 3) for s, v in stages.items() if v[1]},
        "refine_mode": {binding.REFINE_TABLES: "tables", binding.REFINE_DIRECT: "direct", binding.REFINE_SPLIT: "split"}[
            binding.search_refine_mode(w.m, w.dsub, w.b, w.Q, w.r, refine_mode)],
        "setup_s": round(setup_s, 2),
    }

    if headline:
        # What a kernel that reads the code array once reaches on this device, and pass one in the
        # configuration where it really is bound by that stream: a single tile of 16 queries, every
        # code read from HBM once (context for `roofline`, not part of `value`).
        out["hbm_stream_read_gbs"] = round(binding.stream_read_gbs(codes.view(torch.uint8).view(-1)), 1)
        if w.m == 8:
            qtab_v, _, _ = binding.build_small_tables(queries[:16].contiguous(), derived, codes, w.r)
            ws_v = torch.empty(binding.scan_workspace_bytes(w.N, w.m, 16, w.r), dtype=torch.uint8, device=dev)

            def one_tile():
                binding.scan_candidates(codes, qtab_v, w.r, workspace=ws_v, mode=binding.SCAN_TILE16)
            _, st_v = timed(one_tile, 3, 1, binding, torch)
            ms_v = st_v["scan_fast"][0] / st_v["scan_fast"][1]
            gbs = w.N * code_bytes / (ms_v * 1e-3) / 1e9
            out["scan_single_tile"] = {
                "queries": 16, "query_tile": 16, "passes": 1, "bound": "hbm", "achieved": round(gbs, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4),
                "frac_of_stream_read": round(gbs / out["hbm_stream_read_gbs"], 4), "avg_launch_ms": round(ms_v, 4),
                "bytes_per_launch": w.N * code_bytes, "traffic": committed_traffic("scan_fast_single_tile", w.name)}
            del ws_v, qtab_v

    if ms_per_step < 5.0:
        # a step this short is mostly launch latency (25 kernels); the calls are capture-safe, so a caller that
        # repeats a shape can replay a graph: reported beside `value`, which stays the eager figure
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            step()
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.synchronize()
        reps = 20
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        out["graph_replay_ms_per_step"] = round((time.perf_counter() - t0) / reps * 1e3, 3)
        del graph

    if args.compare:
        out["comparison"] = compare_plain(w, cb, codes, queries, ms_per_step, steps, warmup, binding, torch)

    if with_cpu:
        import oracle
        threads = oracle.num_threads()
        cb_np, codes_np = synth.to_numpy(cb), synth.to_numpy(codes)
        der_np = oracle.derive_codebooks(cb_np)
        nsample = min(w.Q, 2 * threads)
        for attempt in range(2):
            q_np = synth.to_numpy(queries)[:nsample]
            t0 = time.perf_counter()
            ref = oracle.search_flat(cb_np, der_np, codes_np, q_np, w.r, w.k)
            cpu_s = time.perf_counter() - t0
            # the headline sample is grown once to about 10 s of oracle work
            grown = min(w.Q, int(nsample * 10.0 / max(cpu_s, 1e-3)) // threads * threads)
            if not headline or attempt or grown <= nsample:
                break
            nsample = grown
        got = synth.to_numpy(ids)[:nsample]
        out["cpu_baseline"] = {
            "value": round(nsample / cpu_s, 3), "unit": "queries/s", "cores": threads, "kind": "oracle",
            "sample": "%d queries of the batch at full N=%d, one query per thread" % (nsample, w.N),
            "seconds": round(cpu_s, 2),
            "result_ids_equal_fraction": float((got == ref["ids"]).mean()),
        }
    del data, cb, codes, queries, ws
    torch.cuda.empty_cache()
    return out


def compare_plain(w, cb, codes, queries, two_pass_ms, steps, warmup, binding, torch):
    """The conventional single-pass search (Alg. 1) on the same device, as context for the two-pass
    figure (the shape of Table 1 and of the Sec. 4.3 slow-down ratios): once over the same 16-bit
    codes with the full tables, once over an 8-bit product quantizer of the same code size (2m
    sub-quantizers of 256 centroids, random codebook and codes: timing only).  Both comparison
    kernels are plain and untuned."""
    dev = queries.device
    Q, k = w.Q, w.k
    batch = min(Q, 256)            # the 16-bit tables of a batch: 256 KiB x m per query
    ws16 = torch.empty(binding.plain_workspace_bytes(w.N, batch, k), dtype=torch.uint8, device=dev)

    def plain16():
        for q0 in range(0, Q, batch):
            qs = queries[q0:q0 + batch]
            binding.plain_search(binding.build_tables(qs, cb), codes, k, ws16)
    e16, st16 = timed(plain16, steps, warmup, binding, torch)

    m8, dsub8 = 2 * w.m, w.dsub // 2
    g = torch.Generator(device=dev); g.manual_seed(w.seed + 8)
    cb8 = 0.3 * torch.randn((m8, 256, dsub8), generator=g, device=dev, dtype=torch.float32)
    codes8 = torch.empty((w.N, m8), dtype=torch.uint8, device=dev)
    flat = codes8.view(-1)
    for s0 in range(0, flat.numel(), 1 << 28):
        e0 = min(flat.numel(), s0 + (1 << 28))
        flat[s0:e0] = torch.randint(0, 256, (e0 - s0,), generator=g, device=dev, dtype=torch.uint8)
    ws8 = torch.empty(binding.plain_workspace_bytes(w.N, Q, k), dtype=torch.uint8, device=dev)

    def plain8():
        binding.plain_search(binding.build_tables_n(queries, cb8), codes8, k, ws8)
    e8, st8 = timed(plain8, steps, warmup, binding, torch)
    ms16, ms8 = e16 / steps * 1e3, e8 / steps * 1e3
    return {
        "two_pass_16bit_ms": round(two_pass_ms, 3),
        "plain_16bit_ms": round(ms16, 3), "plain_16bit_scan_ms": round(st16["plain_scan"][0] / steps, 3),
        "plain_8bit_ms": round(ms8, 3), "plain_8bit_scan_ms": round(st8["plain_scan"][0] / steps, 3),
        "plain_8bit_shape": "PQ %dx8, dsub %d" % (m8, dsub8),
        "two_pass_over_plain_8bit": round(two_pass_ms / ms8, 3),
        "plain_16bit_over_plain_8bit": round(ms16 / ms8, 3),
        "plain_16bit_over_two_pass": round(ms16 / two_pass_ms, 3),
    }


def run_ivf(w, args, steps, warmup, with_cpu):
    import numpy as np
    import torch
    from paper_1905_06900_amd import binding, synth
    dev = "cuda:0"
    t0 = time.perf_counter()
    d = synth.make_ivf(w, dev)
    cb, coarse, offsets, codes, queries = d["codebooks"], d["coarse"], d["offsets"], d["codes"], d["queries"]
    derived = binding.derive_codebooks(cb)                       # index build, not timed
    plane = binding.pack_low_bytes(codes)                        # index build: the bytes pass one reads
    ws = torch.empty(binding.ivf_search_workspace_bytes(w.Q, w.nlist, w.nprobe, w.m, w.r), dtype=torch.uint8, device=dev)
    ids = torch.empty((w.Q, w.k), dtype=torch.uint32, device=dev)
    dist = torch.empty((w.Q, w.k), dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    setup_s = time.perf_counter() - t0

    def step():
        binding.ivf_search(queries, coarse, cb, derived, codes, offsets, w.nprobe, w.r, w.k, plane=plane,
                           workspace=ws, ids=ids, dist=dist)

    if args.calibration_copy:
        calibration_copy(binding, torch, dev)
    elapsed, stages = timed(step, steps, warmup, binding, torch)
    qps = w.Q * steps / elapsed
    # codes in the probed lists of the batch: what one pass of the scan streams (no two queries share them)
    probe = binding.ivf_probe(queries, coarse, w.nprobe).long()
    probed_codes = int((offsets[probe + 1] - offsets[probe]).sum().item())
    dom = max((s for s in stages if s != "misc" and stages[s][1]), key=lambda s: stages[s][0])
    dom_ms, dom_launches = stages[dom]
    if dom == "ivf_scan":
        roofline = hbm_roofline(dom, float(probed_codes) * w.m, dom_ms, dom_launches, steps, w.name,
                                "the stream of low bytes of the probed lists from HBM (lane = code, byte gathers from LDS)",
                                {"probed_codes_per_step": probed_codes, "bytes_per_code": w.m})
    else:
        roofline = {"bound": "alu", "kernel": dom, "achieved": None, "peak": None, "unit": None, "frac": None,
                    "traffic": None, "avg_launch_ms": round(dom_ms / dom_launches, 4)}
    out = {
        "value": round(qps, 2), "unit": "queries/s", "ms_per_step": round(elapsed / steps * 1e3, 3),
        "config": {"workload": w.name, "N": w.N, "queries": w.Q, "m": w.m, "dsub": w.dsub, "r": w.r, "k": w.k,
                   "nlist": w.nlist, "nprobe": w.nprobe, "code_bytes": 2 * w.m, "scan_reads": "low-byte plane",
                   "seed": w.seed},
        "roofline": roofline,
        "stage_ms_per_step": {s: round(v[0] / steps, 3) for s, v in stages.items() if v[1]},
        "setup_s": round(setup_s, 2),
    }
    if with_cpu:
        # The oracle walks only the probed lists: it gets a compact copy of the lists the sample's
        # queries probe (lists renumbered, ids = positions in the compact array) and the library's
        # own probe lists.
        import oracle
        threads = oracle.num_threads()
        nsample = min(w.Q, 8 * threads)
        pr = probe[:nsample]
        lists = torch.unique(pr)
        sizes = offsets[lists + 1] - offsets[lists]
        off_c = torch.zeros(lists.numel() + 1, dtype=torch.int64, device=dev)
        off_c[1:] = torch.cumsum(sizes, 0)
        idx = torch.repeat_interleave(offsets[lists] - off_c[:-1], sizes) + torch.arange(int(off_c[-1]), device=dev)
        # (gathered in pieces: one indexing call over more than ~50 M rows of this 8 G-element array came back wrong)
        codes_c = torch.empty((idx.numel(), w.m), dtype=torch.int16, device=dev)
        for s0 in range(0, idx.numel(), 1 << 24):
            codes_c[s0:s0 + (1 << 24)] = codes.view(torch.int16)[idx[s0:s0 + (1 << 24)]]
        codes_c = codes_c.view(torch.uint16)
        remap = torch.full((w.nlist,), -1, dtype=torch.int64, device=dev)
        remap[lists] = torch.arange(lists.numel(), device=dev)
        cb_np, der_np = synth.to_numpy(cb), oracle.derive_codebooks(synth.to_numpy(cb))
        args_np = (cb_np, der_np, synth.to_numpy(codes_c), off_c.cpu().numpy(), synth.to_numpy(coarse[lists]),
                   synth.to_numpy(queries[:nsample]), remap[pr].to(torch.int32).cpu().numpy(), w.r, w.k)
        t0 = time.perf_counter()
        ref = oracle.search_ivf(*args_np)
        cpu_s = time.perf_counter() - t0
        back = (idx.cpu().numpy())[np.minimum(ref["ids"].astype(np.int64), idx.numel() - 1)]
        got = synth.to_numpy(ids)[:nsample]
        out["cpu_baseline"] = {
            "value": round(nsample / cpu_s, 3), "unit": "queries/s", "cores": threads, "kind": "oracle",
            "sample": "%d queries of the batch over their own %d probed lists (%d codes), one query per thread"
                      % (nsample, int(lists.numel()), int(off_c[-1])),
            "seconds": round(cpu_s, 2),
            "result_ids_equal_fraction": float((got.astype(np.int64) == back).mean()),
        }
    del d, cb, codes, queries, plane, ws
    torch.cuda.empty_cache()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--cfg", type=int, default=None, help="workload index in BASELINE.json (default: 2, the headline, "
                    "with the four others measured briefly beside it)")
    ap.add_argument("--n", type=int, default=None, help="override database size (experiments only)")
    ap.add_argument("--q", type=int, default=None, help="override query batch (experiments only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="headline workload only")
    ap.add_argument("--chunk", type=int, default=0, help="queries per chunk of the fused search (0 = default)")
    ap.add_argument("--refine", choices=("auto", "tables", "direct", "split"), default="auto",
                    help="pass two of the flat workloads: table entries on demand (direct: one kernel; split: by "
                         "sub-quantizer), from full tables, or the library's own choice")
    ap.add_argument("--compare", action="store_true",
                    help="also time the conventional single-pass search (plain 16-bit and plain 8-bit PQ, Alg. 1) "
                         "on the same workload; flat workloads only")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also launch one 1 GiB calibration_copy_kernel (for scaling rocprofv3 --pmc traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import torch
    from paper_1905_06900_amd import binding, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    binding.lib()
    torch.cuda.set_device(0)
    cfg = 2 if args.cfg is None else args.cfg
    w = synth.scaled(synth.WORKLOADS[cfg], N=args.n, Q=args.q)
    with_cpu = not args.no_cpu_baseline
    if w.kind == "flat":
        res = run_flat(w, args, args.steps, args.warmup, with_cpu, headline=True)
    else:
        res = run_ivf(w, args, args.steps, args.warmup, with_cpu)
    out = {
        "metric": METRIC, "value": res.pop("value"), "unit": res.pop("unit"), "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": res.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u8 scan / f32 refine", "data": "synthetic",
    }
    out.update(res)

    if args.cfg is None and not args.no_others and args.n is None and args.q is None:
        others = []
        for c in (0, 1, 3, 4):
            wo = synth.WORKLOADS[c]
            try:
                if wo.kind == "flat":
                    r = run_flat(wo, args, 3, 1, with_cpu, headline=False)
                else:
                    r = run_ivf(wo, args, 3, 1, with_cpu)
                r["steps"] = 3
            except Exception as e:      # never let a side measurement take the headline line down
                r = {"config": {"workload": wo.name}, "error": "%s: %s" % (type(e).__name__, e)}
                torch.cuda.empty_cache()
            others.append(r)
        out["other_workloads"] = others
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())

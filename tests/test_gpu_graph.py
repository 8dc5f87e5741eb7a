"""The search calls only enqueue kernels (no allocation, no memset nodes, no host synchronization), so a
caller may capture them into a HIP graph.  Every replay is compared with the eager result, with eager work
and synchronizations between the replays."""
import numpy as np
import pytest
import torch

from paper_1905_06900_amd import binding, synth
from parity import to_np

pytestmark = pytest.mark.gpu

DEV = "cuda"


@pytest.mark.parametrize("cfg,N,Q,r", [(0, 120_001, 40, 800), (2, 300_007, 1000, 700)])
def test_flat_search_captured_in_a_graph_replays_to_the_eager_result(cfg, N, Q, r):
    # the second case is large enough for the pilot pass of the scan and for the refinement split by sub-quantizer
    w = synth.scaled(synth.WORKLOADS[cfg], N=N, Q=Q, r=r)
    if cfg == 2:
        assert binding.scan_plan(w.N, w.m, w.Q, w.r)["pilot_every"] == 16
        assert binding.search_refine_mode(w.m, w.dsub, 16, w.Q, w.r) == binding.REFINE_SPLIT
    print("graph capture: flat search, cfg%d recipe, N=%d Q=%d r=%d" % (cfg, w.N, w.Q, w.r), flush=True)
    d = synth.make_flat(w, DEV)
    cb, codes, queries = d["codebooks"], d["codes"], d["queries"]
    derived = binding.derive_codebooks(cb)
    ws = torch.empty(binding.search_workspace_bytes(w.N, w.m, w.Q, w.r), dtype=torch.uint8, device=DEV)
    ids = torch.empty((w.Q, w.k), dtype=torch.uint32, device=DEV)
    dist = torch.empty((w.Q, w.k), dtype=torch.float32, device=DEV)
    want_ids, want_dist = binding.search(queries, cb, derived, codes, w.r, w.k, 0, ws)      # eager (also warms up)
    torch.cuda.synchronize()
    want_ids, want_dist = to_np(want_ids).copy(), to_np(want_dist).copy()

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        binding.search(queries, cb, derived, codes, w.r, w.k, 0, ws, ids, dist)            # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            binding.search(queries, cb, derived, codes, w.r, w.k, 0, ws, ids, dist)
    torch.cuda.synchronize()
    for replay in range(4):
        ids.view(torch.int32).fill_(-1)
        dist.fill_(-1.0)
        ws.random_(0, 255)                                    # the call may not depend on what the workspace held
        other = binding.search(queries[:7].contiguous(), cb, derived, codes, w.r, w.k)     # eager work in between
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(to_np(ids), want_ids, err_msg="replay %d ids" % replay)
        np.testing.assert_array_equal(to_np(dist), want_dist, err_msg="replay %d distances" % replay)
        np.testing.assert_array_equal(to_np(other[0]), want_ids[:7])

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


def test_flat_search_captured_in_a_graph_replays_to_the_eager_result():
    w = synth.scaled(synth.WORKLOADS[0], N=120_001, Q=40, r=800)
    print("graph capture: flat search N=%d Q=%d" % (w.N, w.Q), flush=True)
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

"""The small-problem paths (one kernel per entry point, no sort, no workspace)
captured into a HIP graph: every replay must give what the eager calls give.
Replays are interleaved with eager work and synchronisations, as a training
loop would interleave them."""
import numpy as np
import pytest
import torch

import oracle
import workloads
import paper_2108_02191_amd as robe

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
TINY = 1e-30


def bits_equal(a, b):
    return np.array_equal(np.ascontiguousarray(a).ravel().view(np.int32), np.ascontiguousarray(b).ravel().view(np.int32))


@pytest.mark.parametrize("name", ["kaggle_z4", "tiny"])
def test_graph_replays_of_a_small_step_match_eager_calls(name):
    w = workloads.get(name)
    B, F = w.batch, w.n_features
    h = robe.robe_init_hash(w.hash_seed, w.m, w.d, w.Z, w.use_sign)
    H = oracle.init_hash(w.hash_seed, w.m, w.d, w.Z, w.use_sign)
    assert robe.robe_workspace_bytes(h, B, F, B * F) == 0          # the direct scatter: nothing to sort
    M0 = workloads.make_array(w.m, 0)
    G = workloads.make_grad_out(w, 2)
    # static buffers the graph reads and writes
    Md = torch.from_numpy(M0).to(DEV)
    idd = torch.zeros((B, F), dtype=torch.int64, device=DEV)
    Gd = torch.from_numpy(G).to(DEV)
    out = torch.empty((B, F, w.d), dtype=torch.float32, device=DEV)
    ga = torch.zeros(w.m, dtype=torch.float32, device=DEV)
    lr = 0.5

    def step():
        robe.robe_forward(h, Md, idd, None, B, F, out=out)
        robe.robe_backward(h, Gd, idd, None, B, F, ga)
        robe.robe_sgd_update(h, Md, ga, lr)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                      # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    Md.copy_(torch.from_numpy(M0))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    torch.cuda.synchronize()
    Md.copy_(torch.from_numpy(M0))                  # capture runs nothing, but be explicit

    M_ref = M0.copy()
    for k in range(4):
        ids, _ = workloads.make_indices(w, 10 + k)
        idd.copy_(torch.from_numpy(ids))
        graph.replay()
        torch.cuda.synchronize()
        got_out = out.cpu().numpy()
        got_M = Md.cpu().numpy()
        # eager work between the replays (and the expected values): the oracle on the same inputs
        want_out = oracle.forward(H, M_ref, ids, None, B, F)
        assert bits_equal(got_out, want_out), k
        g, S = oracle.backward(H, G, ids, None, B, F)
        step_ref = M_ref.astype(np.float64) - lr * g
        assert np.all(np.abs(got_M.astype(np.float64) - step_ref) <= lr * 1e-5 * S + 1e-6 * np.abs(M_ref) + TINY), k
        assert not ga.cpu().numpy().any()           # the update cleared the gradient inside the graph
        # some unrelated eager launches on the default stream, then continue from the GPU's own state
        scratch = torch.zeros(w.m, dtype=torch.float32, device=DEV)
        robe.robe_backward(h, Gd, idd, None, B, F, scratch)
        torch.cuda.synchronize()
        M_ref = got_M.copy()

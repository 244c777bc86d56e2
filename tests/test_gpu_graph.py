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


@pytest.mark.parametrize("fused", [False, True])
def test_graph_replays_of_a_sorted_backward_match_eager_calls(fused):
    # Large enough for the sorted routes (token sort, combine, then atomics or the region route): they
    # record kernels only, so the whole training step can be captured.  Small-integer gradients make
    # the scatter exact, so every replay must reproduce the eager result bit for bit.
    opt = robe.options(fused_route=robe.ROUTE_REGIONS)
    m, d, Z, B, F = 3_000_017, 128, 32, 12_000, 26
    h = robe.robe_init_hash(5, m, d, Z, 1)
    H = oracle.init_hash(5, m, d, Z, 1)
    rng = np.random.default_rng(0)
    assert robe.robe_workspace_bytes(h, B, F, B * F) > 0
    M0 = rng.standard_normal(m).astype(np.float32)
    G = rng.integers(-3, 4, size=(B, F, d)).astype(np.float32)
    Md = torch.from_numpy(M0).to(DEV)
    st = torch.zeros(m, dtype=torch.float32, device=DEV)
    ga = torch.zeros(m, dtype=torch.float32, device=DEV)
    idd = torch.zeros((B, F), dtype=torch.int64, device=DEV)
    Gd = torch.from_numpy(G).to(DEV)
    out = torch.empty((B, F, d), dtype=torch.float32, device=DEV)
    need = max(robe.robe_workspace_bytes(h, B, F, B * F, opt), robe.robe_fused_workspace_bytes(h, B, F, B * F, opt))
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)

    def step():
        robe.robe_forward(h, Md, idd, None, B, F, out=out)
        if fused:
            robe.robe_backward_adagrad(h, Gd, idd, None, B, F, Md, st, 0.01, 1e-8, workspace=ws, options=opt)
        else:
            robe.robe_backward(h, Gd, idd, None, B, F, ga, workspace=ws, options=opt)
            robe.robe_adagrad_update(h, Md, st, ga, 0.01, 1e-8)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    torch.cuda.synchronize()

    for k in range(3):
        ids = rng.integers(0, 50_000, size=(B, F), dtype=np.int64)
        ids[rng.random((B, F)) < 0.2] = 3
        idd.copy_(torch.from_numpy(ids))
        Md.copy_(torch.from_numpy(M0))
        st.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got_M, got_s, got_out = Md.cpu().numpy(), st.cpu().numpy(), out.cpu().numpy()
        # the same step, eagerly, from the same state
        Md.copy_(torch.from_numpy(M0))
        st.zero_()
        step()
        torch.cuda.synchronize()
        assert bits_equal(got_out, out.cpu().numpy()), k
        assert bits_equal(got_M, Md.cpu().numpy()) and bits_equal(got_s, st.cpu().numpy()), k
        # and against the oracle: exact gradient, so the accumulator is its square
        g, _ = oracle.backward(H, G, ids, None, B, F, threads=8, want_abs=False)
        assert np.array_equal(got_s.astype(np.float64), (g.astype(np.float32) ** 2).astype(np.float64)), k

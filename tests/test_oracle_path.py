"""Pins for the oracle's forward, backward and optimizer step.

Forward and backward are checked against the explicit sketching matrix of
Section 4 (one +-1 per row) built with arbitrary-precision integers on tiny
inputs, against direct circular reads, and against invariants that hold at
any size.  The optimizer step is checked against torch.optim.Adagrad on CPU.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads
from tests import brute

P = 2**31 - 1


def _tiny_case(seed, m, d, Z, sign, B, F, card=50):
    H = oracle.init_hash(seed, m, d, Z, sign)
    rng = np.random.default_rng(seed)
    ids = rng.integers(0, card, size=(B, F))
    M = rng.standard_normal(m).astype(np.float32)
    return H, ids, M


CASES = [(1, 37, 16, 8, 1), (2, 37, 16, 8, 0), (3, 64, 16, 4, 1), (4, 16, 16, 16, 1),
         (5, 101, 12, 1, 1), (6, 8, 16, 8, 0), (7, 1000, 6, 3, 1)]


@pytest.mark.parametrize("seed,m,d,Z,sign", CASES)
def test_single_hot_forward_equals_direct_circular_reads(seed, m, d, Z, sign):
    B, F = 4, 3
    H, ids, M = _tiny_case(seed, m, d, Z, sign, B, F)
    out = oracle.forward(H, M, ids, None, B, F)
    for b in range(B):
        for f in range(F):
            want = brute.embedding(H.coef, P, M, d, Z, sign, f, int(ids[b, f]))
            assert out[b, f].tobytes() == np.array(want, dtype=np.float32).tobytes()


def test_forward_of_identity_array_is_the_index_map():
    # M[j] = j is exact in float32 for j < 2^24, so the output IS idx(e,x,i)
    m, d, Z, B, F = 4099, 16, 4, 8, 5
    H = oracle.init_hash(17, m, d, Z, 0)
    ids = np.random.default_rng(0).integers(0, 10**6, size=(B, F))
    out = oracle.forward(H, np.arange(m, dtype=np.float32), ids, None, B, F)
    for b in range(B):
        for f in range(F):
            assert out[b, f].astype(np.int64).tolist() == brute.position_map(H.coef, P, m, d, Z, f, int(ids[b, f]))


def test_negative_zero_and_sign_flip_are_exact():
    m, d, Z = 16, 16, 16
    H = oracle.init_hash(4, m, d, Z, 1)
    M = np.zeros(m, dtype=np.float32)
    M[::2] = -0.0
    out = oracle.forward(H, M, np.array([[3]]), None, 1, 1)[0, 0]
    pos = brute.position_map(H.coef, P, m, d, Z, 0, 3)
    for i in range(d):
        neg_in = np.signbit(M[pos[i]])
        flip = brute.g(H.coef, P, 1, 0, 3, i) < 0
        assert np.signbit(out[i]) == (neg_in != flip)


def _random_bags(rng, rows, card, mean=3.0):
    sizes = rng.poisson(mean, size=rows)
    sizes[0] = 0                         # always include an empty bag
    off = np.zeros(rows + 1, dtype=np.int64)
    np.cumsum(sizes, out=off[1:])
    ids = rng.integers(0, card, size=int(off[-1]))
    return ids, off


@pytest.mark.parametrize("seed,m,d,Z,sign", CASES)
def test_forward_and_backward_equal_the_sketching_matrix(seed, m, d, Z, sign):
    # forward = S M (bag rows summed), backward = S^T G, S built by brute force
    B, F = 3, 4
    rng = np.random.default_rng(100 + seed)
    H = oracle.init_hash(seed, m, d, Z, sign)
    M = rng.standard_normal(m).astype(np.float32)
    ids, off = _random_bags(rng, B * F, 40)
    tokens = []
    bag_of = []
    for k in range(B * F):
        for t in range(off[k], off[k + 1]):
            tokens.append((k % F, int(ids[t])))
            bag_of.append(k)
    S = brute.sketch_matrix(H.coef, P, m, d, Z, sign, tokens)
    assert np.all((S != 0).sum(axis=1) == 1)                  # exactly one +-1 per row
    per_token = (S @ M.astype(np.float64)).reshape(len(tokens), d)
    want = np.zeros((B * F, d))
    for t, k in enumerate(bag_of):
        want[k] += per_token[t]
    out = oracle.forward(H, M, ids, off, B, F).reshape(B * F, d)
    np.testing.assert_allclose(out, want.astype(np.float32), rtol=0, atol=0)
    assert not out[0].any() and not np.signbit(out[0]).any()    # empty bag -> +0.0

    G = rng.standard_normal((B, F, d)).astype(np.float32)
    g_tok = G.reshape(B * F, d)[bag_of].astype(np.float64).ravel()
    want_ga = S.T @ g_tok
    ga, ab = oracle.backward(H, G, ids, off, B, F)
    np.testing.assert_allclose(ga, want_ga, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(ab, np.abs(S).T @ np.abs(g_tok), rtol=1e-13, atol=1e-13)
    # adjoint identity <S M, G> = <M, S^T G>
    lhs = float((want * G.reshape(B * F, d)).sum())
    assert abs(lhs - float(M.astype(np.float64) @ ga)) <= 1e-9 * (1 + abs(lhs))


def test_forward_and_backward_with_blocks_larger_than_the_embedding():
    # Z > d: forward reads the brute-force positions, backward is its transpose
    B, F, m, d, Z = 4, 3, 211, 4, 16
    for sign in (0, 1):
        H = oracle.init_hash(5 + sign, m, d, Z, sign)
        rng = np.random.default_rng(sign)
        ids = rng.integers(0, 40, size=(B, F))
        M = rng.standard_normal(m).astype(np.float32)
        out = oracle.forward(H, M, ids, None, B, F)
        S = np.zeros((B * F * d, m))
        for b in range(B):
            for f in range(F):
                for i in range(d):
                    pos = brute.position_big_block(H.coef, P, m, d, Z, f, int(ids[b, f]), i)
                    sg = brute.g(H.coef, P, sign, f, int(ids[b, f]), i)
                    S[(b * F + f) * d + i, pos] = sg
                    assert out[b, f, i] == np.float32(sg) * M[pos]
        G = rng.standard_normal((B, F, d)).astype(np.float32)
        ga, _ = oracle.backward(H, G, ids, None, B, F)
        np.testing.assert_allclose(ga, S.T @ G.astype(np.float64).ravel(), rtol=1e-13, atol=1e-13)


def test_single_hot_backward_equals_transposed_jacobian():
    B, F, m, d, Z = 5, 3, 53, 8, 4
    H = oracle.init_hash(77, m, d, Z, 1)
    rng = np.random.default_rng(3)
    ids = rng.integers(0, 6, size=(B, F))                      # few tokens: many duplicates
    tokens = [(f, int(ids[b, f])) for b in range(B) for f in range(F)]
    S = brute.sketch_matrix(H.coef, P, m, d, Z, 1, tokens)
    G = rng.standard_normal((B, F, d)).astype(np.float32)
    ga, _ = oracle.backward(H, G, ids, None, B, F)
    np.testing.assert_allclose(ga, S.T @ G.astype(np.float64).ravel(), rtol=1e-13, atol=1e-13)


def test_bag_of_one_equals_single_hot_and_bag_sum_equals_sum_of_rows():
    w = workloads.get("tiny")
    H = oracle.init_hash(5, 4096, 16, 4, 1)
    M = workloads.make_array(4096, 0)
    B, F = 6, w.n_features
    rng = np.random.default_rng(8)
    ids1 = rng.integers(0, 1000, size=(B, F))
    single = oracle.forward(H, M, ids1, None, B, F)
    as_bags = oracle.forward(H, M, ids1.ravel(), np.arange(B * F + 1), B, F)
    assert single.tobytes() == as_bags.tobytes()

    ids, off = _random_bags(rng, B * F, 1000, mean=4.0)
    pooled = oracle.forward(H, M, ids, off, B, F).reshape(B * F, 16)
    for k in range(B * F):
        toks = ids[off[k]:off[k + 1]]
        if toks.size == 0:
            assert not pooled[k].any()
            continue
        # each token looked up on its own, as feature k % F: put it in column k % F of a 1-sample batch
        acc = np.zeros(16)
        for x in toks:
            row = np.zeros((1, F), dtype=np.int64)
            row[0, k % F] = x
            acc += oracle.forward(H, M, row, None, 1, F)[0, k % F].astype(np.float64)
        assert np.array_equal(pooled[k], acc.astype(np.float32))
        # order inside a bag does not matter beyond rounding
        perm = ids.copy()
        perm[off[k]:off[k + 1]] = toks[::-1]
        again = oracle.forward(H, M, perm, off, B, F).reshape(B * F, 16)[k]
        np.testing.assert_allclose(again, pooled[k], rtol=1e-6, atol=1e-9)


def test_backward_mass_conservation_without_sign():
    # sign off: every gradient element lands in exactly one slot
    w = workloads.get("tiny")
    H = oracle.init_hash(w.hash_seed, w.m, w.d, w.Z, 0)
    ids, _ = workloads.make_indices(w, 1)
    G = workloads.make_grad_out(w, 2)
    ga, ab = oracle.backward(H, G, ids, None, w.batch, w.n_features)
    assert abs(ga.sum() - G.astype(np.float64).sum()) < 1e-8
    assert abs(ab.sum() - np.abs(G.astype(np.float64)).sum()) < 1e-8
    # bags: a row's gradient is delivered once per token of its bag
    rng = np.random.default_rng(1)
    idsb, off = _random_bags(rng, w.rows, 1000)
    gab, _ = oracle.backward(H, G, idsb, off, w.batch, w.n_features)
    sizes = np.diff(off).astype(np.float64)
    want = (G.reshape(w.rows, w.d).astype(np.float64).sum(axis=1) * sizes).sum()
    assert abs(gab.sum() - want) < 1e-7


def test_backward_threads_do_not_change_the_result_beyond_rounding():
    H = oracle.init_hash(1, 5000, 16, 4, 1)
    rng = np.random.default_rng(2)
    ids = rng.integers(0, 30, size=(64, 4))
    G = rng.standard_normal((64, 4, 16)).astype(np.float32)
    a, _ = oracle.backward(H, G, ids, None, 64, 4, threads=1)
    b, _ = oracle.backward(H, G, ids, None, 64, 4, threads=4)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-12)


def test_forward_threads_give_the_same_bits_as_the_sequential_loop():
    # the full-size GPU comparisons use the threaded oracle: rows are independent, so the split over
    # threads must not change a single bit (single-hot and bags, sign on and off, a ragged row count)
    rng = np.random.default_rng(3)
    for sign in (0, 1):
        H = oracle.init_hash(7 + sign, 5003, 16, 4, sign)
        M = rng.standard_normal(5003).astype(np.float32)
        M[::5] = -0.0
        ids = rng.integers(0, 300, size=(67, 5))
        a = oracle.forward(H, M, ids, None, 67, 5, threads=1)
        for t in (2, 4, 7):
            b = oracle.forward(H, M, ids, None, 67, 5, threads=t)
            assert np.array_equal(a.view(np.int32), b.view(np.int32)), (sign, t)
        idsb, off = _random_bags(rng, 67 * 5, 300)
        a = oracle.forward(H, M, idsb, off, 67, 5, threads=1)
        for t in (2, 4, 7):
            b = oracle.forward(H, M, idsb, off, 67, 5, threads=t)
            assert np.array_equal(a.view(np.int32), b.view(np.int32)), (sign, t)


def test_adagrad_matches_torch_cpu_and_touches_only_nonzero_gradients():
    rng = np.random.default_rng(0)
    n = 4096
    M0 = rng.standard_normal(n).astype(np.float32)
    p = torch.nn.Parameter(torch.from_numpy(M0.astype(np.float64)))
    opt = torch.optim.Adagrad([p], lr=0.01, eps=1e-8, initial_accumulator_value=0.0, lr_decay=0.0)
    M, s = M0.copy(), np.zeros(n, dtype=np.float32)
    ref_M = M0.astype(np.float64)
    for step in range(3):
        g = rng.standard_normal(n).astype(np.float32)
        g[rng.random(n) < 0.5] = 0.0                 # half the slots untouched this step
        before_M, before_s = M.copy(), s.copy()
        p.grad = torch.from_numpy(g.astype(np.float64))
        opt.step()
        grad = g.copy()
        oracle.adagrad(M, s, grad, 0.01, 1e-8)
        assert not grad.any()                         # consumed and zeroed
        untouched = g == 0
        assert np.array_equal(M[untouched], before_M[untouched])
        assert np.array_equal(s[untouched], before_s[untouched])
        # torch keeps float64 state; ours is stored in float32 after every step
        np.testing.assert_allclose(M, p.detach().numpy(), rtol=2e-6, atol=2e-7)
        np.testing.assert_allclose(s, opt.state[p]["sum"].numpy(), rtol=1e-6)
    assert not np.array_equal(M, M0)
    del ref_M


def test_adagrad_first_step_closed_form():
    # from s = 0: M' = M - lr * g / (|g| + eps)
    g = np.array([0.5, -2.0, 0.0, 1e-3], dtype=np.float32)
    M = np.array([1.0, 1.0, 1.0, 1.0], dtype=np.float32)
    s = np.zeros(4, dtype=np.float32)
    oracle.adagrad(M, s, g.copy(), 0.01, 1e-8)
    want = 1.0 - 0.01 * g.astype(np.float64) / (np.abs(g.astype(np.float64)) + 1e-8)
    np.testing.assert_allclose(M, want.astype(np.float32), rtol=0, atol=0)
    np.testing.assert_allclose(s, (g.astype(np.float64) ** 2).astype(np.float32), rtol=0, atol=0)


def test_sgd_matches_torch_cpu_and_closed_form():
    rng = np.random.default_rng(1)
    n = 2048
    M0 = rng.standard_normal(n).astype(np.float32)
    p = torch.nn.Parameter(torch.from_numpy(M0.astype(np.float64)))
    opt = torch.optim.SGD([p], lr=1.0)                 # the paper's DLRM setting (Appendix: SGD, lr 1.0)
    M = M0.copy()
    for step in range(3):
        g = rng.standard_normal(n).astype(np.float32)
        g[rng.random(n) < 0.5] = 0.0
        before = M.copy()
        p.grad = torch.from_numpy(g.astype(np.float64))
        opt.step()
        grad = g.copy()
        oracle.sgd(M, grad, 1.0)
        assert not grad.any()
        assert np.array_equal(M[g == 0], before[g == 0])
        want = (before.astype(np.float64) - 1.0 * g.astype(np.float64)).astype(np.float32)
        assert np.array_equal(M, want)                 # one rounding of the exact result
        np.testing.assert_allclose(M, p.detach().numpy(), rtol=1e-6, atol=1e-6)


def test_inner_product_estimator_is_unbiased_over_hash_draws():
    # Theorem 1 (Section 4.1): E<x^, y^> = <x, y> for the signed projection.
    # Loose Monte-Carlo check over seeds; it fails if the sign or the block
    # placement were systematically wrong.
    n_tok, d, Z, m = 6, 8, 4, 64
    rng = np.random.default_rng(0)
    X = rng.standard_normal((n_tok, d)).astype(np.float32)
    Y = (X + 0.5 * rng.standard_normal((n_tok, d))).astype(np.float32)
    true = float((X.astype(np.float64) * Y).sum())
    ids = np.arange(n_tok).reshape(n_tok, 1)
    est = []
    for seed in range(400):
        H = oracle.init_hash(seed, m, d, Z, 1)
        xh, _ = oracle.backward(H, X.reshape(n_tok, 1, d), ids, None, n_tok, 1, want_abs=False)
        yh, _ = oracle.backward(H, Y.reshape(n_tok, 1, d), ids, None, n_tok, 1, want_abs=False)
        est.append(float(xh @ yh))
    est = np.array(est)
    assert abs(est.mean() - true) < 4 * est.std() / np.sqrt(len(est)) + 1e-9


# ---------------------------------------------------------------------------------------------
# Tables of different dimensions sharing the array (Section 3.2, "Multiple embedding tables")
# ---------------------------------------------------------------------------------------------
MIXED = [(11, 101, (8, 4, 16, 4), 4, 1), (12, 37, (16, 8, 8), 8, 0), (13, 64, (3, 6, 9, 3), 3, 1),
         (14, 50, (5, 1, 2), 1, 1), (15, 16, (16, 16), 16, 0)]


@pytest.mark.parametrize("seed,m,dims,Z,sign", MIXED)
def test_mixed_dimensions_are_per_table_embeddings_side_by_side(seed, m, dims, Z, sign):
    # every table's slice of a sample's row is that table's embedding, built from the two-piece
    # circular reads of the forward equation with d = dims[f]
    F, B = len(dims), 5
    H = oracle.init_hash(seed, m, max(dims), Z, sign)
    rng = np.random.default_rng(seed)
    ids = rng.integers(0, 40, size=(B, F))
    M = rng.standard_normal(m).astype(np.float32)
    out = oracle.forward_mixed(H, dims, M, ids, None, B)
    assert out.shape == (B, sum(dims))
    col = np.concatenate([[0], np.cumsum(dims)])
    for b in range(B):
        for f in range(F):
            want = brute.embedding(H.coef, P, M, dims[f], Z, sign, f, int(ids[b, f]))
            assert out[b, col[f]:col[f + 1]].tobytes() == np.array(want, dtype=np.float32).tobytes()


@pytest.mark.parametrize("seed,m,dims,Z,sign", MIXED)
def test_mixed_forward_and_backward_equal_the_sketching_matrix(seed, m, dims, Z, sign):
    # rows of S: one per (sample, table, element) in output order; forward = S M, backward = S^T G
    F, B = len(dims), 3
    H = oracle.init_hash(seed, m, max(dims), Z, sign)
    rng = np.random.default_rng(seed + 100)
    flat = rng.integers(0, 30, size=40)
    sizes = rng.integers(0, 4, size=B * F)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    flat = flat[:off[-1]]
    M = rng.standard_normal(m).astype(np.float32)
    D = sum(dims)
    S = np.zeros((B * D, m))
    col = np.concatenate([[0], np.cumsum(dims)])
    for b in range(B):
        for f in range(F):
            k = b * F + f
            toks = [(f, int(x)) for x in flat[off[k]:off[k + 1]]]
            if toks:
                St = brute.sketch_matrix(H.coef, P, m, dims[f], Z, sign, toks)      # (len * d_f) x m
                S[b * D + col[f]: b * D + col[f + 1]] = St.reshape(len(toks), dims[f], m).sum(axis=0)
    out = oracle.forward_mixed(H, dims, M, flat, off, B)
    assert np.allclose(out.ravel(), S @ M.astype(np.float64), rtol=0, atol=1e-6)
    G = rng.standard_normal((B, D)).astype(np.float32)
    ga, ab = oracle.backward_mixed(H, dims, G, flat, off, B)
    assert np.allclose(ga, S.T @ G.ravel().astype(np.float64), rtol=0, atol=1e-12)
    assert np.allclose(ab, np.abs(S).T @ np.abs(G.ravel().astype(np.float64)), rtol=0, atol=1e-12)


def test_mixed_with_equal_dimensions_is_the_uniform_path():
    H = oracle.init_hash(3, 997, 8, 4, 1)
    rng = np.random.default_rng(3)
    B, F = 6, 4
    ids = rng.integers(0, 100, size=(B, F))
    M = rng.standard_normal(997).astype(np.float32)
    G = rng.standard_normal((B, F, 8)).astype(np.float32)
    assert oracle.forward_mixed(H, [8] * F, M, ids, None, B).tobytes() == oracle.forward(H, M, ids, None, B, F).tobytes()
    ga, ab = oracle.backward_mixed(H, [8] * F, G, ids, None, B)
    gu, au = oracle.backward(H, G, ids, None, B, F)
    assert np.array_equal(ga, gu) and np.array_equal(ab, au)
    with pytest.raises(ValueError):
        oracle.forward_mixed(H, [8, 6], M, ids[:, :2], None, B)      # 6 is neither a multiple nor a divisor of 4


# ---------------------------------------------------------------------------------------------
# bfloat16 array
# ---------------------------------------------------------------------------------------------
def _torch_bf16_bits(a: np.ndarray) -> np.ndarray:
    return torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def test_bf16_rounding_matches_the_library_conversion_and_the_format_rules():
    rng = np.random.default_rng(0)
    vals = [0.0, -0.0, 1.0, -1.0, 1.00390625, 1.01171875, 3.4028235e38, 1e-40, -1e-45, np.inf, -np.inf,
            0.01, -0.01, 65280.0, 65408.0, 2.0 ** -126, 2.0 ** -133]
    a = np.array(vals, dtype=np.float32)
    # exact ties: patterns whose dropped half is 0x8000, on even and odd kept halves; and neighbours
    ties = np.array([0x3F808000, 0x3F818000, 0x3F807FFF, 0x3F808001, 0x7F7F8000, 0x00008000, 0x00018000,
                     0x80008000, 0xBF808000, 0x7F7FFFFF], dtype=np.uint32).view(np.float32)
    big = rng.standard_normal(200_000).astype(np.float32) * np.float32(0.01)
    bits = rng.integers(0, 2**32, size=200_000, dtype=np.uint64).astype(np.uint32).view(np.float32)
    bits = bits[~np.isnan(bits)]
    for arr in (a, ties, big, bits):
        got = oracle.to_bf16(arr)
        assert np.array_equal(got, _torch_bf16_bits(np.ascontiguousarray(arr)))
    # hand-checked rules: tie to even, carry into the exponent, NaN stays NaN
    assert oracle.to_bf16(np.array([0x3F808000], dtype=np.uint32).view(np.float32))[0] == 0x3F80    # tie, even kept
    assert oracle.to_bf16(np.array([0x3F818000], dtype=np.uint32).view(np.float32))[0] == 0x3F82    # tie, odd kept -> up
    assert oracle.to_bf16(np.array([0x3FFFFFFF], dtype=np.uint32).view(np.float32))[0] == 0x4000    # carries into the exponent
    assert oracle.to_bf16(np.array([0x7F7FFFFF], dtype=np.uint32).view(np.float32))[0] == 0x7F80    # overflows to infinity
    nan = oracle.to_bf16(np.array([0x7F800001, 0xFFC12345], dtype=np.uint32).view(np.float32))
    assert all((int(h) & 0x7F80) == 0x7F80 and (int(h) & 0x007F) != 0 for h in nan)


@pytest.mark.parametrize("seed,m,d,Z,sign", CASES)
def test_forward_on_a_bf16_array_is_the_forward_of_the_widened_array(seed, m, d, Z, sign):
    # widening is exact, so the bf16 forward must equal the (pinned) float32 forward of the array
    # that a library conversion produces from the same bit patterns
    B, F = 4, 3
    H, ids, M = _tiny_case(seed, m, d, Z, sign, B, F)
    Mb = oracle.to_bf16(M)
    widened = torch.from_numpy(Mb.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    assert oracle.forward_bf16(H, Mb, ids, None, B, F).tobytes() == oracle.forward(H, widened, ids, None, B, F).tobytes()
    rng = np.random.default_rng(seed)
    sizes = rng.integers(0, 5, size=B * F)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    flat = rng.integers(0, 50, size=int(off[-1]))
    assert oracle.forward_bf16(H, Mb, flat, off, B, F).tobytes() == oracle.forward(H, widened, flat, off, B, F).tobytes()
    # and quantisation moves every element by at most half a bf16 ulp: 2^-9 relative
    assert np.all(np.abs(widened - M) <= np.abs(M) * 2.0 ** -8)

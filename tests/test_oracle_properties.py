"""Property tests of the oracle over random shapes (hypothesis): whatever
(m, d, Z, sign, ids) are drawn, the C oracle agrees with the arbitrary-precision
restatement of the paper's formulas and keeps the invariants of Section 3."""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
from tests import brute

P = 2**31 - 1


@st.composite
def shapes(draw):
    Z = draw(st.sampled_from([1, 2, 3, 4, 5, 8, 16]))
    C = draw(st.integers(1, 4))
    d = Z * C
    m = draw(st.integers(Z, 300))
    sign = draw(st.integers(0, 1))
    seed = draw(st.integers(0, 2**64 - 1))
    return m, d, Z, sign, seed


ids_strategy = st.one_of(st.integers(0, 10**6), st.integers(-(2**63), 2**63 - 1),
                         st.sampled_from([0, P - 1, P, P + 1, 2**62, 2**63 - 1, -1]))


@settings(max_examples=150, deadline=None)
@given(shapes(), st.lists(ids_strategy, min_size=1, max_size=6), st.integers(1, 5))
def test_forward_equals_brute_force_embedding(shape, ids, F):
    m, d, Z, sign, seed = shape
    H = oracle.init_hash(seed, m, d, Z, sign)
    B = len(ids)
    idm = np.array([[ids[b]] * F for b in range(B)], dtype=np.int64)
    M = np.random.default_rng(seed % 2**32).standard_normal(m).astype(np.float32)
    out = oracle.forward(H, M, idm, None, B, F)
    for b in range(B):
        for f in range(F):
            want = brute.embedding(H.coef, P, M, d, Z, sign, f, int(idm[b, f]))
            assert out[b, f].tobytes() == np.array(want, dtype=np.float32).tobytes()
            pos = [oracle.idx(H, f, int(idm[b, f]), i) for i in range(d)]
            assert all(0 <= q < m for q in pos)
            for c in range(d // Z):
                assert len(set(pos[c * Z:(c + 1) * Z])) == Z


@settings(max_examples=60, deadline=None)
@given(shapes(), st.integers(1, 4), st.integers(1, 3), st.integers(0, 2**32 - 1))
def test_backward_is_the_adjoint_of_forward(shape, B, F, data_seed):
    m, d, Z, sign, seed = shape
    H = oracle.init_hash(seed, m, d, Z, sign)
    rng = np.random.default_rng(data_seed)
    sizes = rng.integers(0, 4, size=B * F)
    off = np.zeros(B * F + 1, dtype=np.int64)
    np.cumsum(sizes, out=off[1:])
    ids = rng.integers(0, 20, size=int(off[-1]), dtype=np.int64)
    M = rng.standard_normal(m).astype(np.float32)
    G = rng.standard_normal((B, F, d)).astype(np.float32)
    out = oracle.forward(H, M, ids, off, B, F).astype(np.float64)
    ga, ab = oracle.backward(H, G, ids, off, B, F)
    # <forward(M), G> = <M, backward(G)>; forward is rounded once per element, hence the tolerance
    lhs = float((out * G).sum())
    rhs = float(M.astype(np.float64) @ ga)
    assert abs(lhs - rhs) <= 1e-6 * (float(np.abs(M).astype(np.float64) @ ab) + 1e-12)
    if not sign:
        want = float((G.reshape(B * F, d).astype(np.float64).sum(axis=1) * sizes).sum())
        assert abs(float(ga.sum()) - want) <= 1e-9 * (1 + float(ab.sum()))

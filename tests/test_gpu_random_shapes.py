"""Randomised GPU parity: many small problems with shapes, sizes, sign, bag
structure and id ranges drawn from a fixed seed, each checked against the
oracle to the bars of the parity suite.  The draws cover what the fixed cases
may miss: odd batch and table counts, arrays barely larger than a block,
embeddings sharing a block (Z > d), bags from empty to hundreds of tokens,
negative and huge ids, both row orders and every scatter strategy; the
bfloat16 array and tables of mixed dimensions ride along on the same draws."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2108_02191_amd as robe

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
THREADS = max(1, min(16, os.cpu_count() or 1))


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def draw_case(rng):
    kind = rng.integers(0, 5)
    if kind == 0:       # power-of-two shapes: the tiled kernels
        d = int(2 ** rng.integers(0, 9))
        Z = int(2 ** rng.integers(0, int(np.log2(d)) + 1))
    elif kind == 1:     # arbitrary divisors: lane groups wider than the row; beyond d = 512 the shape-generic kernel
        Z = int(rng.integers(1, 13))
        d = Z * int(rng.integers(1, 9)) * int(rng.choice([1, 1, 1, 7, 11]))
    elif kind == 2:     # Z > d
        d = int(rng.integers(1, 17))
        Z = d * int(rng.integers(2, 9))
    elif kind == 3:     # three, six or eight elements per lane
        d = int(rng.choice([24, 48, 96, 192, 384, 512]))
        divs = [z for z in range(1, d + 1) if d % z == 0]
        Z = int(rng.choice(divs))
    else:               # the benchmark's shape family
        d, Z = 128, int(rng.choice([1, 8, 32, 128]))
    m = int(rng.choice([Z, Z + 1, 2 * Z + 3, 1000 + Z, 65_537 + Z, 1_000_003 + Z]))
    B = int(rng.choice([1, 2, 7, 33, 130]))
    F = int(rng.choice([1, 2, 5, 26, 40]))
    sign = int(rng.integers(0, 2))
    return m, d, Z, B, F, sign


def draw_ids(rng, n):
    mode = rng.integers(0, 3)
    if mode == 0:
        return rng.integers(0, 50, size=n, dtype=np.int64)            # heavy repetition
    if mode == 1:
        return rng.integers(0, 4 * 10**7, size=n, dtype=np.int64)
    return rng.integers(-(2**63), 2**63 - 1, size=n, dtype=np.int64)  # any 64-bit pattern


@pytest.mark.parametrize("chunk", range(8))
def test_random_problems_match_the_oracle(chunk):
    rng = np.random.default_rng(1000 + chunk)
    for case in range(12):
        m, d, Z, B, F, sign = draw_case(rng)
        opt = robe.options(row_order=int(rng.choice([robe.ROWS_MEMORY, robe.ROWS_BY_TABLE_ALWAYS])),
                           backward_route=int(rng.choice([robe.ROUTE_DIRECT, robe.ROUTE_COMBINE, robe.ROUTE_REGIONS])),
                           tile_combine=int(rng.choice([1, 2])))
        repro = robe.options(reproducible=1)
        tag = f"chunk {chunk} case {case}: m={m} d={d} Z={Z} B={B} F={F} sign={sign}"
        print(tag, flush=True)
        seed = int(rng.integers(0, 2**63))
        h = robe.robe_init_hash(seed, m, d, Z, sign)
        H = oracle.init_hash(seed, m, d, Z, sign)
        assert tuple(h.coef) == H.coef, tag
        M = rng.standard_normal(m).astype(np.float32)
        rows = B * F
        # single-hot
        ids = draw_ids(rng, rows).reshape(B, F)
        out = robe.robe_forward(h, dev(M), dev(ids), None, B, F, options=opt).cpu().numpy()
        want = oracle.forward(H, M, ids, None, B, F, threads=THREADS)
        assert np.array_equal(out.view(np.int32), want.view(np.int32)), tag
        # bags
        sizes = rng.poisson(rng.choice([0.5, 3.0, 20.0]), size=rows).astype(np.int64)
        if rows > 2 and rng.random() < 0.5:
            sizes[int(rng.integers(0, rows))] = int(rng.integers(100, 400))
        off = np.zeros(rows + 1, dtype=np.int64)
        np.cumsum(sizes, out=off[1:])
        idsb = draw_ids(rng, int(off[-1]))
        outb = robe.robe_forward(h, dev(M), dev(idsb), dev(off), B, F, options=opt).cpu().numpy()
        wantb = oracle.forward(H, M, idsb, off, B, F, threads=THREADS)
        H_abs = oracle.Hash(H.m, H.d, H.Z, 0, H.P, H.coef)
        S = oracle.forward(H_abs, np.abs(M), idsb, off, B, F, threads=THREADS).astype(np.float64)
        assert np.all(np.abs(outb.astype(np.float64) - wantb) <= 1e-5 * S + 1e-30), tag
        # backward, small-integer gradients: exact in any order
        Gi = rng.integers(-3, 4, size=(B, F, d)).astype(np.float32)
        for (i_, o_) in ((ids, None), (idsb, off)):
            ga = torch.zeros(m, dtype=torch.float32, device=DEV)
            robe.robe_backward(h, dev(Gi), dev(i_), dev(o_), B, F, ga, options=opt)
            ref, _ = oracle.backward(H, Gi, i_, o_, B, F, threads=1)
            assert np.array_equal(ga.cpu().numpy().astype(np.float64), ref), tag
            # the same call with the reproducible option gives the same sums (exact here) when it has a route
            gr = torch.zeros(m, dtype=torch.float32, device=DEV)
            try:
                robe.robe_backward(h, dev(Gi), dev(i_), dev(o_), B, F, gr, options=repro)
            except robe.RobeError as e:
                assert "reproducible" in str(e), tag          # shapes without an atomic-free route
            else:
                assert np.array_equal(gr.cpu().numpy().astype(np.float64), ref), tag
        # bfloat16 array: single-hot bit-exact
        Mb = oracle.to_bf16(M)
        outq = robe.robe_forward_bf16(h, dev(Mb.view(np.int16)), dev(ids), None, B, F).cpu().numpy()
        wantq = oracle.forward_bf16(H, Mb, ids, None, B, F)
        assert np.array_equal(outq.view(np.int32), wantq.view(np.int32)), tag
        # tables of mixed dimensions (multiples of Z), single-hot forward bit-exact, backward exact
        if Z <= 64:
            dims = [int(Z * rng.integers(1, 5)) for _ in range(F)]
            if rng.random() < 0.3:                                    # some tables narrower than the block
                divs = [z for z in range(1, Z + 1) if Z % z == 0]
                dims[0] = int(rng.choice(divs))
            if F > 2:
                dims[1] = dims[0]                                     # a run of equal dimensions
            outm = robe.robe_forward_mixed(h, dims, dev(M), dev(ids), None, B, options=opt).cpu().numpy()
            wantm = oracle.forward_mixed(H, dims, M, ids, None, B)
            assert np.array_equal(outm.view(np.int32), wantm.view(np.int32)), tag
            Gm = rng.integers(-3, 4, size=(B, sum(dims))).astype(np.float32)
            gm = torch.zeros(m, dtype=torch.float32, device=DEV)
            robe.robe_backward_mixed(h, dims, dev(Gm), dev(idsb), dev(off), B, gm, options=opt)
            refm, _ = oracle.backward_mixed(H, dims, Gm, idsb, off, B)
            assert np.array_equal(gm.cpu().numpy().astype(np.float64), refm), tag
            # the reproducible option: the region route over all tables, or a loud refusal (a table
            # narrower than the block, a shape without that route)
            gq = torch.zeros(m, dtype=torch.float32, device=DEV)
            try:
                robe.robe_backward_mixed(h, dims, dev(Gm), dev(idsb), dev(off), B, gq, options=repro)
            except robe.RobeError as e:
                assert "reproducible" in str(e), tag
            else:
                assert min(dims) >= Z or idsb.size == 0, tag      # (no tokens: nothing to do, any shape)
                assert np.array_equal(gq.cpu().numpy().astype(np.float64), refm), tag

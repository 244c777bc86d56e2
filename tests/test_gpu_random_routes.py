"""Randomised GPU parity of the sorted backward routes at sizes where regions, record kernels and the
lookup in the sorted list all get real work: shapes (Z <= d, Z > d, three-element lanes), array sizes
from 50 thousand to 67 million slots, routes, record variants, region sizes, sort key bits, the
reproducible option, the fused step and tables of mixed dimensions are drawn from a fixed seed;
small-integer gradients make every float32 sum exact, so the comparison with the oracle is bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2108_02191_amd as robe
from tests import test_gpu_mixed_dims as MD
from tests import test_gpu_parity as P

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.mark.parametrize("seed", range(24))
def test_random_sorted_routes_match_the_oracle(seed):
    rng = np.random.default_rng(seed)
    kind = rng.integers(0, 4)
    if kind == 0:
        d = int(2 ** rng.integers(3, 8)); Z = int(2 ** rng.integers(0, int(np.log2(d)) + 1))
    elif kind == 1:       # Z > d
        d = int(2 ** rng.integers(2, 7)); Z = d * int(rng.choice([2, 3, 4, 8]))
    elif kind == 2:
        d = int(rng.choice([24, 48, 96, 192])); Z = int(rng.choice([z for z in (8, 24, 48, 96) if d % z == 0 or z % d == 0]))
    else:
        d, Z = 128, int(rng.choice([8, 32, 128]))
    m = int(rng.choice([50_021, 300_007, 1_000_003, 5_000_011, 2**26 + 3, 45_000_007]))
    m = max(m, Z)
    sign = int(rng.integers(0, 2))
    F = int(rng.choice([3, 8, 26]))
    B = int(rng.choice([40, 300, 1500]))
    card = int(rng.choice([30, 3000, 10**6]))
    route = int(rng.choice([robe.ROUTE_COMBINE, robe.ROUTE_REGIONS, robe.ROUTE_REGIONS]))
    fields = dict(backward_route=route, region_records=int(rng.integers(0, 3)), region_shift=int(rng.choice([0, 0, 10, 13, 14])))
    if rng.random() < 0.3:
        fields["key_bits"] = int(rng.choice([8, 12, 16, 24, 31]))
    repro = rng.random() < 0.3
    tag = f"seed {seed}: m={m} d={d} Z={Z} sign={sign} B={B} F={F} card={card} {fields} repro={repro}"
    print(tag, flush=True)
    h, H = P.both_hashes(seed * 7 + 1, m, d, Z, sign)
    bags = rng.random() < 0.5
    if bags:
        ids, off = P.random_bags(rng, B * F, card, 6.0, long_bag=int(rng.choice([0, 500])))
    else:
        ids, off = rng.integers(0, card, size=(B, F), dtype=np.int64), None
        ids[rng.random((B, F)) < 0.2] = 5
    Gi = rng.integers(-3, 4, size=(B, F, d)).astype(np.float32)
    opts = [robe.options(**fields)]
    if repro:
        opts.append(robe.options(reproducible=1, region_records=fields["region_records"]))
    ref, _ = oracle.backward(H, Gi, ids, off, B, F, threads=8)
    for o in opts:
        ga = torch.zeros(m, dtype=torch.float32, device=DEV)
        try:
            robe.robe_backward(h, P.to_dev(Gi), P.to_dev(ids), P.to_dev(off), B, F, ga, options=o)
        except robe.RobeError as e:
            assert "reproducible" in str(e), tag
            continue
        assert np.array_equal(ga.cpu().numpy().astype(np.float64), ref), tag
    # fused
    fo = robe.options(fused_route=int(rng.choice([robe.ROUTE_AUTO, robe.ROUTE_REGIONS, robe.ROUTE_TWO_STEP])),
                      region_records=fields["region_records"], region_shift=fields["region_shift"])
    P._check_fused(h, H, Gi, ids, off, B, F, m, options=fo)
    # tables of mixed dimensions on the same ids
    if Z <= d and Z <= 64 and not bags:
        dims = [int(Z * rng.integers(1, 5)) for _ in range(F)]
        hm, Hm = MD.hashes(seed + 3, m, Z, sign, max(dims))
        Gm = rng.integers(-3, 4, size=(B, sum(dims))).astype(np.float32)
        refm, _ = oracle.backward_mixed(Hm, dims, Gm, ids, None, B)
        for o in (robe.options(backward_route=route, region_records=fields["region_records"]), robe.options(reproducible=1)):
            gm = torch.zeros(m, dtype=torch.float32, device=DEV)
            try:
                robe.robe_backward_mixed(hm, dims, MD.dev(Gm), MD.dev(ids), None, B, gm, options=o)
            except robe.RobeError as e:
                assert "reproducible" in str(e), tag
                continue
            assert np.array_equal(gm.cpu().numpy().astype(np.float64), refm), tag
        MD._fused_mixed_check(hm, Hm, dims, Gm, ids, None, B, m, robe.options(fused_route=int(rng.choice([0, 3]))))

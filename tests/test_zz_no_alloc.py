"""The entry point that allocates nothing (robe_backward_noalloc): called through the C ABI, its
result is compared with robe_backward's on the same inputs, to the parity bar of the backward pass
(bit for bit with small-integer gradients, where every summation order gives the same floats; within
1e-5 * S of the oracle with real-valued ones), on two calls in a row that share the built-in
workspace, the second with a smaller input.  It must pass alone in a fresh process and after every
other test."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2108_02191_amd as robe

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
TINY = 1e-30


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def call_noalloc(h, Gd, idd, offd, n, B, F, ga, opt):
    """Straight through ctypes: device pointers and sizes, nothing else."""
    rc = robe.lib().robe_backward_noalloc(ctypes.byref(h), Gd.data_ptr(), idd.data_ptr(),
                                          None if offd is None else offd.data_ptr(), n, B, F, ga.data_ptr(),
                                          None if opt is None else ctypes.byref(opt),
                                          torch.cuda.current_stream().cuda_stream)
    assert rc == robe.ROBE_OK, robe.lib().robe_last_error()


@pytest.mark.parametrize("route", [robe.ROUTE_COMBINE, robe.ROUTE_REGIONS, robe.ROUTE_DIRECT])
@pytest.mark.parametrize("sign", [0, 1])
def test_noalloc_backward_matches_the_workspace_entry_point_on_two_calls_in_a_row(route, sign):
    m, d, Z, F = 1_000_003, 64, 16, 26
    h = robe.robe_init_hash(77 + sign, m, d, Z, sign)
    H = oracle.init_hash(77 + sign, m, d, Z, sign)
    opt = robe.options(backward_route=route)
    rng = np.random.default_rng(route * 2 + sign)
    limit = int(robe.lib().robe_noalloc_max_workspace_bytes())
    assert limit == 32 << 20
    for B in (1500, 200):                                   # the second call is the smaller one
        ids = rng.integers(0, 20_000, size=(B, F), dtype=np.int64)
        ids[rng.random((B, F)) < 0.2] = 3                   # a frequent token: long runs
        need = robe.robe_workspace_bytes(h, B, F, ids.size, opt)
        assert need <= limit and (need > 0) == (route != robe.ROUTE_DIRECT)
        for bags in (False, True):
            if bags:
                sizes = rng.poisson(1.0, size=B * F).astype(np.int64)
                off = np.zeros(B * F + 1, dtype=np.int64)
                np.cumsum(sizes, out=off[1:])
                flat = rng.integers(0, 5000, size=int(off[-1]), dtype=np.int64)
                assert robe.robe_workspace_bytes(h, B, F, flat.size, opt) <= limit
            else:
                flat, off = ids, None
            idd, offd = dev(flat), dev(off)
            # small-integer gradients: the two entry points must agree bit for bit, and with the oracle
            Gi = rng.integers(-3, 4, size=(B, F, d)).astype(np.float32)
            Gd = dev(Gi)
            a = torch.zeros(m, dtype=torch.float32, device=DEV)
            b = torch.zeros(m, dtype=torch.float32, device=DEV)
            call_noalloc(h, Gd, idd, offd, flat.size, B, F, a, opt)
            robe.robe_backward(h, Gd, idd, offd, B, F, b, options=opt)
            ref, _ = oracle.backward(H, Gi, flat, off, B, F)
            got = a.cpu().numpy()
            assert np.array_equal(got.view(np.int32), b.cpu().numpy().view(np.int32)), (B, bags)
            assert np.array_equal(got.astype(np.float64), ref), (B, bags)
            # real-valued gradients: both within the backward pass's tolerance of the oracle
            G = rng.standard_normal((B, F, d)).astype(np.float32)
            Gd = dev(G)
            a.zero_()
            call_noalloc(h, Gd, idd, offd, flat.size, B, F, a, opt)
            ref, S = oracle.backward(H, G, flat, off, B, F)
            err = np.abs(a.cpu().numpy().astype(np.float64) - ref)
            assert np.all(err <= 1e-5 * S + TINY), (B, bags, float((err / (S + TINY)).max()))


def test_noalloc_backward_rejects_what_does_not_fit_and_needs_no_workspace_for_direct_scatters():
    m, d, Z, F = 25_000_000, 128, 32, 26
    h = robe.robe_init_hash(1, m, d, Z, 0)
    B = 65536                                               # 1.7 M tokens: 27 MB of sort buffers fit ...
    assert robe.robe_workspace_bytes(h, B, F, B * F) <= 32 << 20
    B = 131072                                              # ... 3.4 M tokens do not
    need = robe.robe_workspace_bytes(h, B, F, B * F)
    assert need > 32 << 20
    fake = ctypes.c_void_p(256)                             # validation fails before anything is read
    rc = robe.lib().robe_backward_noalloc(ctypes.byref(h), fake, fake, None, B * F, B, F, fake, None, None)
    assert rc == robe.ROBE_EINVAL and b"built-in" in robe.lib().robe_last_error()

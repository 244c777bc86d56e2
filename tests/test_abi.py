"""Host-side checks of the C-ABI library: it loads, exports what the header
declares, draws the documented coefficients, and turns bad arguments into
error codes before anything touches a GPU.  No compute call is made here."""
import ctypes
import os
import re

import pytest

import oracle
import paper_2108_02191_amd as robe

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "robe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(robe_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = robe.lib()
    names = _declared_symbols()
    assert set(names) == set(robe.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_header_is_plain_c():
    # the boundary is a C ABI: the header must compile as C99 on its own
    import subprocess
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c",
                        os.path.join(ROOT, "include", "robe.h")], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_struct_layout_matches_header():
    # uint64 m; uint32 d, Z, use_sign, P; 8 x uint32 coefficients
    assert ctypes.sizeof(robe.RobeHash) == 8 + 4 * 4 + 8 * 4
    assert robe.RobeHash.m.offset == 0 and robe.RobeHash.d.offset == 8 and robe.RobeHash.Ah.offset == 24
    # robe_options_t: the fields the header lists, in its order, sixteen int32 in all
    text = open(os.path.join(ROOT, "include", "robe.h")).read()
    body = re.search(r"typedef struct robe_options_t \{(.*?)\} robe_options_t;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = [n.strip().split("[")[0] for decl in body.split(";") if decl.strip()
             for n in decl.replace("int32_t", "").replace("void", "").replace("*", "").split(",")]
    assert names == [f[0] for f in robe.RobeOptions._fields_]
    assert ctypes.sizeof(robe.RobeOptions) == 16 * 4 + 2 * ctypes.sizeof(ctypes.c_void_p)


@pytest.mark.parametrize("seed", [0, 1, 7, 2**40 + 3, 2**64 - 1])
def test_init_hash_draws_the_same_coefficients_as_the_oracle(seed):
    h = robe.robe_init_hash(seed, 25_000_000, 128, 32, 1)
    o = oracle.init_hash(seed, 25_000_000, 128, 32, 1)
    assert tuple(h.coef) == o.coef
    assert (h.m, h.d, h.Z, h.use_sign, h.P) == (o.m, o.d, o.Z, 1, o.P)


@pytest.mark.parametrize("m,d,Z", [(0, 16, 4), (2**31, 16, 4), (100, 16, 5), (100, 0, 1), (100, 16, 0), (8, 16, 16)])
def test_init_hash_rejects_bad_shapes(m, d, Z):
    with pytest.raises(robe.RobeError) as ei:
        robe.robe_init_hash(0, m, d, Z, 0)
    assert ei.value.code == robe.ROBE_EINVAL


def test_entry_points_reject_bad_arguments_without_a_gpu():
    L = robe.lib()
    h = robe.robe_init_hash(1, 1000, 16, 4, 0)
    ref = ctypes.byref(h)
    fake = ctypes.c_void_p(256)  # never dereferenced: validation fails first
    EINVAL = robe.ROBE_EINVAL
    # null hash
    assert L.robe_forward(None, fake, fake, None, 4, 2, 2, fake, None, None) == EINVAL
    assert b"hash" in L.robe_last_error()
    # negative batch, bad feature count, single-hot size mismatch
    assert L.robe_forward(ref, fake, fake, None, 4, -1, 2, fake, None, None) == EINVAL
    assert L.robe_forward(ref, fake, fake, None, 4, 2, 0, fake, None, None) == EINVAL
    assert L.robe_forward(ref, fake, fake, None, 5, 2, 2, fake, None, None) == EINVAL
    # null buffers
    assert L.robe_forward(ref, None, fake, None, 4, 2, 2, fake, None, None) == EINVAL
    assert L.robe_forward(ref, fake, None, None, 4, 2, 2, fake, None, None) == EINVAL
    assert L.robe_forward(ref, fake, fake, None, 4, 2, 2, None, None, None) == EINVAL
    assert L.robe_backward(ref, None, fake, None, 4, 2, 2, fake, None, 0, None, None) == EINVAL
    assert L.robe_backward(ref, fake, fake, None, 4, 2, 2, None, None, 0, None, None) == EINVAL
    assert L.robe_adagrad_update(ref, None, fake, fake, 0.01, 1e-8, None) == EINVAL
    assert L.robe_adagrad_update(ref, fake, fake, fake, 0.01, 0.0, None) == EINVAL
    assert L.robe_adagrad_update(ref, fake, fake, fake, float("nan"), 1e-8, None) == EINVAL
    assert L.robe_backward_adagrad(ref, fake, fake, None, 4, 2, 2, None, fake, 0.01, 1e-8, None, 0, None, None) == EINVAL
    assert L.robe_backward_adagrad(ref, fake, fake, None, 4, 2, 2, fake, fake, 0.01, -1.0, None, 0, None, None) == EINVAL
    assert L.robe_backward_adagrad(ref, fake, fake, None, 4, 2, 2, fake, fake, 0.01, 1e-8, None, 0, None, None) == EINVAL  # no workspace
    assert b"workspace" in L.robe_last_error()
    assert L.robe_sgd_update(ref, None, fake, 1.0, None) == EINVAL
    assert L.robe_backward_sgd(ref, fake, fake, None, 4, 2, 2, None, 1.0, None, 0, None, None) == EINVAL
    assert L.robe_backward_sgd(ref, fake, fake, None, 4, 2, 2, fake, float("inf"), None, 0, None, None) == EINVAL
    assert L.robe_backward_sgd(ref, fake, fake, None, 4, 2, 2, fake, 1.0, None, 0, None, None) == EINVAL    # no workspace
    assert L.robe_backward_sgd(ref, None, None, None, 0, 0, 2, fake, 1.0, None, 0, None, None) == robe.ROBE_OK
    assert L.robe_sgd_update(ref, fake, fake, float("inf"), None) == EINVAL
    assert L.robe_offsets(ref, None, 3, 2, fake, None, None) == EINVAL
    assert L.robe_offsets(ref, fake, -3, 2, fake, None, None) == EINVAL
    # corrupted hash structs
    for field, val in [("P", 101), ("Ah", 0), ("Bh", 2**31 - 1), ("Dh", 2**31 - 1), ("Z", 3), ("m", 2**31), ("m", 2)]:
        bad = robe.robe_init_hash(1, 1000, 16, 4, 0)
        setattr(bad, field, val)
        assert L.robe_forward(ctypes.byref(bad), fake, fake, None, 4, 2, 2, fake, None, None) == EINVAL, field
    # tables of mixed dimensions: the dims array is validated on the host
    dims_ok = (ctypes.c_uint32 * 2)(8, 4)
    dims_bad = (ctypes.c_uint32 * 2)(8, 6)
    assert L.robe_forward_mixed(ref, None, fake, fake, None, 4, 2, 2, fake, None, None) == EINVAL
    assert L.robe_forward_mixed(ref, dims_bad, fake, fake, None, 4, 2, 2, fake, None, None) == EINVAL
    assert b"dims[1]" in L.robe_last_error()
    assert L.robe_forward_mixed(ref, dims_ok, None, fake, None, 4, 2, 2, fake, None, None) == EINVAL
    assert L.robe_backward_mixed(ref, dims_ok, fake, fake, None, 5, 2, 2, fake, None, 0, None, None) == EINVAL
    assert L.robe_backward_adagrad_mixed(ref, dims_ok, fake, fake, None, 5, 2, 2, fake, fake, 0.01, 1e-8, None, 0, None, None) == EINVAL
    assert L.robe_backward_adagrad_mixed(ref, dims_bad, fake, fake, None, 4, 2, 2, fake, fake, 0.01, 1e-8, None, 0, None, None) == EINVAL
    need = ctypes.c_size_t(7)
    assert L.robe_fused_mixed_workspace_bytes(ref, dims_ok, 2, 2, 4, None, ctypes.byref(need)) == robe.ROBE_OK and need.value > 0
    assert L.robe_fused_mixed_workspace_bytes(ref, dims_bad, 2, 2, 4, None, ctypes.byref(need)) == EINVAL
    assert L.robe_forward_mixed(ref, dims_ok, None, None, None, 0, 0, 2, None, None, None) == robe.ROBE_OK
    # bfloat16 array
    assert L.robe_forward_bf16(ref, None, fake, None, 4, 2, 2, fake, None, None) == EINVAL
    assert L.robe_forward_bf16(ref, fake, fake, None, 5, 2, 2, fake, None, None) == EINVAL
    assert L.robe_forward_bf16(ref, None, None, None, 0, 0, 2, None, None, None) == robe.ROBE_OK
    assert L.robe_array_to_bf16(None, fake, 8, None) == EINVAL
    assert L.robe_array_to_bf16(None, None, 0, None) == robe.ROBE_OK
    # the sort primitive
    flag = ctypes.c_int(7)
    assert L.robe_sort_pairs(fake, fake, fake, fake, 10, 9, 8, fake, 1 << 20, ctypes.byref(flag), None) == EINVAL
    assert L.robe_sort_pairs(fake, fake, fake, fake, 10, 0, 8, None, 0, ctypes.byref(flag), None) == EINVAL
    assert L.robe_sort_pairs(fake, fake, fake, fake, 10, 0, 8, fake, 1 << 20, None, None) == EINVAL
    assert L.robe_sort_pairs(None, None, None, None, 0, 0, 8, None, 0, ctypes.byref(flag), None) == robe.ROBE_OK and flag.value == 0
    assert L.robe_sort_workspace_bytes(8_500_000) >= 256 * 4 * (8_500_000 // 4096)
    # options are validated before anything else
    bad_opt = robe.options(backward_route=9)
    assert L.robe_forward(ref, fake, fake, None, 4, 2, 2, fake, ctypes.byref(bad_opt), None) == EINVAL
    assert b"options" in L.robe_last_error()
    bad_opt = robe.RobeOptions()
    bad_opt.reserved[1] = 1
    assert L.robe_backward(ref, fake, fake, None, 4, 2, 2, fake, None, 0, ctypes.byref(bad_opt), None) == EINVAL
    # empty problems are no-ops that succeed
    assert L.robe_forward(ref, None, None, None, 0, 0, 2, None, None, None) == robe.ROBE_OK
    assert L.robe_backward(ref, None, None, None, 0, 0, 2, None, None, 0, None, None) == robe.ROBE_OK
    assert L.robe_offsets(ref, None, 0, 2, None, None, None) == robe.ROBE_OK
    # the workspace queries are host arithmetic: a status, and the size through the out-parameter
    need = ctypes.c_size_t(7)
    assert L.robe_workspace_bytes(ref, 4, 2, 8, None, ctypes.byref(need)) == robe.ROBE_OK and need.value == 0
    assert L.robe_workspace_bytes(ref, 4, 2, 8, None, None) == EINVAL
    need.value = 7
    assert L.robe_workspace_bytes(None, 4, 2, 8, None, ctypes.byref(need)) == EINVAL and need.value == 0
    assert L.robe_fused_workspace_bytes(ref, -1, 2, 8, None, ctypes.byref(need)) == EINVAL
    assert L.robe_fused_workspace_bytes(ref, 4, 2, 8, None, ctypes.byref(need)) == robe.ROBE_OK and need.value >= 4 * 1000
    big = robe.robe_init_hash(1, 250_000_000, 128, 32, 0)
    assert L.robe_fused_workspace_bytes(ctypes.byref(big), 16384, 26, 8_500_000, None, ctypes.byref(need)) == robe.ROBE_OK
    assert 16 * 8_500_000 < need.value
    forced = robe.options(backward_route=robe.ROUTE_COMBINE)
    assert L.robe_workspace_bytes(ref, 4, 2, 8, ctypes.byref(forced), ctypes.byref(need)) == robe.ROBE_OK and need.value >= 16 * 8

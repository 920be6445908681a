"""The C-ABI library: it loads, exports what include/meft.h declares, and validates arguments on the
host before touching a device (no GPU needed: every call here is rejected before any launch)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    lib = os.path.join(ROOT, "paper_2406_04984_amd", "libmeft.so")
    if not os.path.exists(lib):
        import __graft_entry__
        __graft_entry__.build()
    from paper_2406_04984_amd import binding
    return binding


def test_every_declared_symbol_is_exported(B):
    header = open(os.path.join(ROOT, "include", "meft.h")).read()
    declared = set(re.findall(r"\b(meft_[a-z_]+)\s*\(", header))
    declared -= {"meft_status", "meft_dtype", "meft_shape", "meft_adam"}
    assert declared == set(B.EXPORTS)
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert getattr(lib, name) is not None


def test_status_strings(B):
    assert B.status_string(0) == "ok"
    assert len({B.status_string(i) for i in range(5)}) == 5


def _shape(B, **kw):
    base = dict(T=16, d=64, n_blocks=4, block_size=8, top_e=2, top_k=4, dtype="f32")
    base.update(kw)
    return B.make_shape(**base)


def test_shape_validation(B):
    assert B.meft_check_shape(_shape(B)) == B.MEFT_OK
    assert B.meft_workspace_bytes(_shape(B)) >= 256
    bad = [dict(top_e=5), dict(top_e=0), dict(top_k=17), dict(top_k=0), dict(T=-1), dict(d=0),
           dict(N=31), dict(dtype=7), dict(activation=1), dict(flags=2), dict(flags=16), dict(block_size=0)]
    for kw in bad:
        s = _shape(B, **kw)
        assert B.meft_check_shape(s) == B.MEFT_ERR_INVALID_ARG, kw
        assert B.meft_workspace_bytes(s) == 0
    for kw in [dict(d=60), dict(d=16392), dict(T=1, block_size=1 << 22, top_e=2, top_k=4, n_blocks=2)]:
        assert B.meft_check_shape(_shape(B, **kw)) == B.MEFT_ERR_UNSUPPORTED, kw
    # 16384 candidates per token: selected from global memory, supported
    assert B.meft_check_shape(_shape(B, block_size=8192, top_e=2, top_k=4, n_blocks=2)) == B.MEFT_OK
    # T*top_k must stay below 2^31
    assert B.meft_check_shape(_shape(B, T=1 << 30, top_k=4)) == B.MEFT_ERR_INVALID_ARG


def test_workspace_grows_with_the_problem(B):
    small = B.meft_workspace_bytes(_shape(B))
    big = B.meft_workspace_bytes(_shape(B, T=4096, d=1024, n_blocks=64, block_size=256, top_e=4, top_k=128,
                                        dtype="bf16"))
    assert big > small
    # the candidate scores dominate: T * top_e * block_size floats
    assert big >= 4096 * 4 * 256 * 4


def test_null_and_misaligned_pointers_are_rejected_before_any_launch(B):
    s = _shape(B)
    need = B.meft_workspace_bytes(s)
    fake = 0x1000  # never dereferenced on the host; every call below must fail validation first
    rc = B._lib.meft_route(ctypes.byref(s), None, fake, None, fake, None, fake, need, None)
    assert rc == B.MEFT_ERR_INVALID_ARG
    rc = B._lib.meft_route(ctypes.byref(s), fake + 4, fake, None, fake, None, fake, need, None)
    assert rc == B.MEFT_ERR_INVALID_ARG
    rc = B._lib.meft_route(ctypes.byref(s), fake, fake, None, fake, None, None, 0, None)
    assert rc == B.MEFT_ERR_WORKSPACE
    rc = B._lib.meft_route(ctypes.byref(s), fake, fake, None, fake, None, fake, need - 1, None)
    assert rc == B.MEFT_ERR_WORKSPACE
    rc = B._lib.meft_route(ctypes.byref(s), fake, fake, None, fake, None, fake + 16, need, None)
    assert rc == B.MEFT_ERR_WORKSPACE
    rc = B._lib.meft_sparse_fwd(ctypes.byref(s), fake, fake, fake, fake, fake, None, fake, fake, need, None)
    assert rc == B.MEFT_ERR_INVALID_ARG
    rc = B._lib.meft_sparse_bwd(ctypes.byref(s), fake, fake, fake, fake, fake, fake, None, fake, fake, fake,
                                None, fake, need, None)
    assert rc == B.MEFT_ERR_INVALID_ARG
    rc = B._lib.meft_sparse_bwd(ctypes.byref(s), fake, fake, fake, fake, fake, fake, None, fake, fake, fake,
                                fake, fake, 8, None)
    assert rc == B.MEFT_ERR_WORKSPACE
    bad = _shape(B, top_e=9)
    rc = B._lib.meft_sparse_fwd(ctypes.byref(bad), fake, fake, fake, fake, fake, fake, fake, fake, need, None)
    assert rc == B.MEFT_ERR_INVALID_ARG
    host_kv = _shape(B, flags=B.MEFT_FLAG_HOST_KV)
    assert B.meft_check_shape(host_kv) == B.MEFT_OK
    assert B.meft_check_shape(_shape(B, flags=B.MEFT_FLAG_HOST_KV | B.MEFT_FLAG_KEEP_STAGED)) == B.MEFT_OK
    assert B.meft_check_shape(_shape(B, flags=4)) == B.MEFT_ERR_INVALID_ARG       # needs MEFT_FLAG_HOST_KV
    assert B.meft_check_shape(_shape(B, flags=7)) == B.MEFT_OK
    assert B.meft_check_shape(_shape(B, flags=9)) == B.MEFT_OK            # host-resident + reuse of the forward's tables
    assert B.meft_check_shape(_shape(B, flags=8)) == B.MEFT_OK
    assert B.meft_check_shape(_shape(B, flags=17)) == B.MEFT_ERR_INVALID_ARG
    fake = 0x1000
    assert B._lib.meft_hostkv_stage(ctypes.byref(_shape(B)), fake, fake, fake, fake, 1 << 30, None) == B.MEFT_ERR_INVALID_ARG
    # the host-resident variant needs room for device copies of K, V and staging for dK, dV
    assert B.meft_workspace_bytes(host_kv) >= B.meft_workspace_bytes(s) + 4 * 32 * 64 * 4


def test_adam_rows_validates_on_the_host(B):
    s = _shape(B)
    fake = 0x1000
    ok = B.MeftAdam(1e-4, 0.9, 0.999, 1e-8, 1)

    def call(shape, hp, W=fake, G=fake, m=fake, v=fake, master=None, touched=fake, n=fake):
        return B._lib.meft_adam_rows(ctypes.byref(shape), ctypes.byref(hp) if hp is not None else None, W, G, m, v,
                                     master, touched, n, None)

    assert call(s, None) == B.MEFT_ERR_INVALID_ARG
    assert call(s, ok, W=None) == B.MEFT_ERR_INVALID_ARG
    assert call(s, ok, m=fake + 8) == B.MEFT_ERR_INVALID_ARG
    assert call(s, ok, master=fake + 4) == B.MEFT_ERR_INVALID_ARG
    assert call(s, ok, n=None) == B.MEFT_ERR_INVALID_ARG
    assert call(s, B.MeftAdam(1e-4, 0.9, 0.999, 1e-8, 0)) == B.MEFT_ERR_INVALID_ARG      # steps count from 1
    assert call(s, B.MeftAdam(1e-4, 1.0, 0.999, 1e-8, 1)) == B.MEFT_ERR_INVALID_ARG      # beta1 < 1
    assert call(s, B.MeftAdam(1e-4, 0.9, -0.1, 1e-8, 1)) == B.MEFT_ERR_INVALID_ARG
    assert call(s, B.MeftAdam(1e-4, 0.9, 0.999, -1.0, 1)) == B.MEFT_ERR_INVALID_ARG
    assert call(s, B.MeftAdam(float("nan"), 0.9, 0.999, 1e-8, 1)) == B.MEFT_ERR_INVALID_ARG
    assert call(_shape(B, flags=B.MEFT_FLAG_HOST_KV), ok) == B.MEFT_ERR_UNSUPPORTED
    assert call(_shape(B, top_e=9), ok) == B.MEFT_ERR_INVALID_ARG


def test_union_calls_validate_on_the_host(B):
    s = _shape(B, dtype="bf16")
    need = B.meft_union_workspace_bytes(s)
    assert need > 0
    fake = 0x1000
    f = B._lib.meft_union_fwd
    assert f(ctypes.byref(s), None, fake, fake, fake, fake, fake, fake, fake, need, None) == B.MEFT_ERR_INVALID_ARG
    assert f(ctypes.byref(s), fake, fake, fake, fake, fake, None, fake, fake, need, None) == B.MEFT_ERR_INVALID_ARG
    assert f(ctypes.byref(s), fake, fake + 2, fake, fake, fake, fake, fake, fake, need, None) == B.MEFT_ERR_INVALID_ARG
    assert f(ctypes.byref(s), fake, fake, fake, fake, fake, fake, fake, None, 0, None) == B.MEFT_ERR_WORKSPACE
    assert f(ctypes.byref(s), fake, fake, fake, fake, fake, fake, fake, fake, need - 1, None) == B.MEFT_ERR_WORKSPACE
    b = B._lib.meft_union_bwd
    assert b(ctypes.byref(s), fake, fake, fake, fake, fake, fake, None, None, fake, fake, need, None) == B.MEFT_ERR_INVALID_ARG
    assert b(ctypes.byref(s), fake, fake, fake, fake, fake, fake, None, fake, fake, fake, need - 1, None) == B.MEFT_ERR_WORKSPACE
    f32 = _shape(B, dtype="f32")
    assert B.meft_union_workspace_bytes(f32) == 0
    assert f(ctypes.byref(f32), fake, fake, fake, fake, fake, fake, fake, fake, 1 << 30, None) == B.MEFT_ERR_UNSUPPORTED


def test_probes_validate_on_the_host(B):
    fake = 0x1000
    assert B._lib.meft_probe_copy(None, fake, 16, None) == B.MEFT_ERR_INVALID_ARG
    assert B._lib.meft_probe_copy(fake, fake + 8, 16, None) == B.MEFT_ERR_INVALID_ARG
    assert B._lib.meft_probe_copy(fake, fake, 24, None) == B.MEFT_ERR_INVALID_ARG
    assert B._lib.meft_probe_mfma(None, 4, 4, None) == B.MEFT_ERR_INVALID_ARG
    assert B._lib.meft_probe_mfma(fake, 0, 4, None) == B.MEFT_ERR_INVALID_ARG
    assert B._lib.meft_probe_mfma(fake, 65537, 4, None) == B.MEFT_ERR_INVALID_ARG
    assert B._lib.meft_probe_mfma(fake, 4, 0, None) == B.MEFT_ERR_INVALID_ARG

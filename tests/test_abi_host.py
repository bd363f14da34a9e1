"""Host-only checks of the C ABI: the library loads, exports every declared
symbol, and rejects bad arguments before any GPU work (no compute calls here)."""
import ctypes
import os
import re

import pytest

from paper_2409_14939_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = "".join(open(os.path.join(ROOT, "include", f)).read()
                   for f in sorted(os.listdir(os.path.join(ROOT, "include"))) if f.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fastgl_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    L = B.lib()
    names = declared_symbols()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_constants_and_sizes():
    assert B.fastgl_long_row_threshold() >= B.fastgl_long_row_chunk() > 0
    small = B.fastgl_block_plan_bytes(10, 10, 10)
    big = B.fastgl_block_plan_bytes(1000, 1000, 100000)
    assert 0 < small < big
    assert B.fastgl_block_workspace_bytes(10, 10, 10, 8, "f32") > small
    assert B.fastgl_block_plan_bytes(-1, 10, 10) == 0
    assert B.fastgl_block_workspace_bytes(10, 10, 10, 0, "f32") == 0


FAKE = ctypes.c_void_p(0x1000)     # aligned, never dereferenced: the calls below fail before any launch


def fwd(indptr=FAKE, indices=FAKE, w=None, nd=4, ns=4, ne=4, feat=8, mode=0, dt=0, X=FAKE, out=FAKE,
        plan=None, ws=FAKE, wsb=1 << 30):
    return B.lib().fastgl_block_aggregate_fwd(indptr, indices, w, nd, ns, ne, feat, mode, dt, X, out, plan,
                                              ws, wsb, None)


@pytest.mark.parametrize("kw,status,text", [
    (dict(nd=-1), B.FASTGL_ERR_INVALID_ARG, "negative"),
    (dict(feat=0), B.FASTGL_ERR_INVALID_ARG, "feat"),
    (dict(mode=3), B.FASTGL_ERR_INVALID_ARG, "mode"),
    (dict(dt=2), B.FASTGL_ERR_INVALID_ARG, "dtype"),
    (dict(indptr=None), B.FASTGL_ERR_INVALID_ARG, "indptr"),
    (dict(indices=None), B.FASTGL_ERR_INVALID_ARG, "indices"),
    (dict(X=None), B.FASTGL_ERR_INVALID_ARG, "NULL"),
    (dict(out=ctypes.c_void_p(0x1002)), B.FASTGL_ERR_INVALID_ARG, "aligned"),
    (dict(ws=None), B.FASTGL_ERR_INVALID_ARG, "workspace"),
    (dict(ws=ctypes.c_void_p(0x1010)), B.FASTGL_ERR_INVALID_ARG, "workspace"),
    (dict(wsb=16), B.FASTGL_ERR_WORKSPACE, "too small"),
    (dict(ns=2 ** 31), B.FASTGL_ERR_UNSUPPORTED, "2^31"),
    (dict(ne=2 ** 31 - 200), B.FASTGL_ERR_UNSUPPORTED, "look-ahead"),      # the kernels read ahead in int32
    (dict(nd=0, ne=3), B.FASTGL_ERR_INVALID_ARG, "at least one"),
])
def test_bad_arguments_are_refused_before_launch(kw, status, text):
    assert fwd(**kw) == status
    assert text in B.fastgl_last_error()


def test_static_scratch_entry_point_checks_on_the_host():
    f = B.lib().fastgl_block_aggregate_fwd_static

    def call(indptr=FAKE, indices=FAKE, w=None, nd=4, ns=4, ne=4, feat=8, mode=0, dt=0, X=FAKE, out=FAKE):
        return f(indptr, indices, w, nd, ns, ne, feat, mode, dt, X, out, None)
    assert call(nd=-1) == B.FASTGL_ERR_INVALID_ARG and "negative" in B.fastgl_last_error()
    assert call(feat=0) == B.FASTGL_ERR_INVALID_ARG
    assert call(X=None) == B.FASTGL_ERR_INVALID_ARG
    assert call(mode=7) == B.FASTGL_ERR_INVALID_ARG
    # sizes beyond the array: refused with both numbers in the text, before any HIP call
    assert call(nd=6_000_000, ns=1, ne=0) == B.FASTGL_ERR_WORKSPACE
    assert "static scratch" in B.fastgl_last_error() and str(B.STATIC_SCRATCH_BYTES) in B.fastgl_last_error()
    assert call(nd=1000, ns=1000, ne=90_000_000, feat=256) == B.FASTGL_ERR_WORKSPACE


def test_layer_entry_point_checks_on_the_host():
    f = B.lib().fastgl_layer_fwd
    assert B.fastgl_layer_fwd_fuses(256, 47, "f32") and B.fastgl_layer_fwd_fuses(4, 64, "f32")
    assert not B.fastgl_layer_fwd_fuses(256, 65, "f32") and not B.fastgl_layer_fwd_fuses(260, 47, "f32")
    assert not B.fastgl_layer_fwd_fuses(30, 16, "f32") and not B.fastgl_layer_fwd_fuses(256, 47, "bf16")

    def call(nd=4, ns=4, ne=4, K=8, mode=0, dt=0, X=FAKE, W=FAKE, bias=None, N=4, H=FAKE, Y=FAKE, ws=FAKE, wsb=1 << 30):
        return f(FAKE, FAKE, None, nd, ns, ne, K, mode, dt, X, W, bias, N, 0, H, Y, None, ws, wsb, None)
    assert call(N=-1) == B.FASTGL_ERR_INVALID_ARG
    assert call(K=0) == B.FASTGL_ERR_INVALID_ARG
    assert call(X=None) == B.FASTGL_ERR_INVALID_ARG
    assert call(W=None) == B.FASTGL_ERR_INVALID_ARG
    assert call(ws=None) == B.FASTGL_ERR_INVALID_ARG
    assert call(wsb=8) == B.FASTGL_ERR_WORKSPACE
    assert call(K=602, H=None) == B.FASTGL_ERR_INVALID_ARG and "two kernels" in B.fastgl_last_error()
    assert call(nd=0, ne=0) == B.FASTGL_OK                                   # no target nodes: nothing to do


def test_plan_and_gather_argument_checks():
    L = B.lib()
    out = ctypes.c_void_p()
    for bad in (0, 4, 6, 7, 9, 13, 16, 20, 32, 33, -1):      # 16 is the short-rows hint: it needs a part to go with
        assert L.fastgl_block_plan_create(FAKE, FAKE, 4, 4, 4, bad, FAKE, 1 << 30, None, ctypes.byref(out)) == B.FASTGL_ERR_INVALID_ARG, bad
    assert L.fastgl_block_plan_create(FAKE, FAKE, 4, 4, 4, 3, FAKE, 8, None, ctypes.byref(out)) == B.FASTGL_ERR_WORKSPACE
    assert L.fastgl_block_plan_create(FAKE, FAKE, 4, 4, 4, 3, None, 1 << 30, None, ctypes.byref(out)) == B.FASTGL_ERR_INVALID_ARG
    assert out.value is None
    assert L.fastgl_block_plan_export(None, None) == B.FASTGL_ERR_INVALID_ARG
    L.fastgl_block_plan_destroy(None)
    assert L.fastgl_gather_rows(FAKE, 10, FAKE, 3, 0, 0, FAKE, None) == B.FASTGL_ERR_INVALID_ARG
    assert L.fastgl_gather_rows(None, 10, FAKE, 3, 8, 0, FAKE, None) == B.FASTGL_ERR_INVALID_ARG
    n = ctypes.c_int64()
    assert L.fastgl_block_validate(FAKE, FAKE, 4, 4, 4, None, ctypes.byref(n), None) == B.FASTGL_ERR_INVALID_ARG


def test_update_argument_checks():
    L = B.lib()
    big = B.fastgl_update_slab_rows(512345, 100, 256)
    assert B.fastgl_update_slab_rows(-1, 4, 4) == 0
    assert 32 <= B.fastgl_update_slab_rows(100, 100, 256) <= B.fastgl_update_slab_rows(91331, 256, 256) <= big <= 2048
    assert all(B.fastgl_update_slab_rows(m, 100, 256) % 32 == 0 for m in (1, 77, 5000, 512345))
    assert B.fastgl_update_bwd_workspace_bytes(-1, 4, 4) == 0
    nslab = -(-512345 // big)
    assert B.fastgl_update_bwd_workspace_bytes(512345, 100, 256) >= 4 * nslab * (100 * 256 + 256)
    assert B.fastgl_update_bwd_workspace_bytes(512345 + big, 100, 256) > B.fastgl_update_bwd_workspace_bytes(512345, 100, 256)
    assert L.fastgl_update_fwd(FAKE, FAKE, None, -1, 4, 4, 0, FAKE, None) == B.FASTGL_ERR_INVALID_ARG
    assert "negative" in B.fastgl_last_error()
    assert L.fastgl_update_fwd(FAKE, FAKE, None, 2 ** 31, 4, 4, 0, FAKE, None) == B.FASTGL_ERR_UNSUPPORTED
    assert L.fastgl_update_fwd(None, FAKE, None, 4, 4, 4, 0, FAKE, None) == B.FASTGL_ERR_INVALID_ARG
    assert L.fastgl_update_fwd(FAKE, FAKE, None, 4, 4, 4, 0, ctypes.c_void_p(0x1002), None) == B.FASTGL_ERR_INVALID_ARG
    assert L.fastgl_update_fwd(FAKE, FAKE, None, 0, 4, 4, 0, None, None) == B.FASTGL_OK      # nothing to do
    bwd = L.fastgl_update_bwd
    assert bwd(FAKE, FAKE, None, FAKE, 4, 4, 4, 1, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == B.FASTGL_ERR_INVALID_ARG
    assert "relu" in B.fastgl_last_error()
    assert bwd(FAKE, FAKE, FAKE, None, 4, 4, 4, 0, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == B.FASTGL_ERR_INVALID_ARG
    assert bwd(FAKE, FAKE, FAKE, FAKE, 4, 4, 4, 0, None, FAKE, None, None, 1 << 30, None) == B.FASTGL_ERR_INVALID_ARG
    assert "workspace" in B.fastgl_last_error()
    assert bwd(FAKE, FAKE, FAKE, FAKE, 4, 4, 4, 0, None, FAKE, None, FAKE, 8, None) == B.FASTGL_ERR_WORKSPACE
    assert bwd(FAKE, FAKE, FAKE, FAKE, 4, 4, 4, 0, None, None, None, None, 0, None) == B.FASTGL_OK   # nothing asked


def test_idmap_argument_checks():
    L = B.lib()
    assert B.fastgl_idmap_table_slots(0) == 1024 and B.fastgl_idmap_table_slots(600) == 1024
    assert B.fastgl_idmap_table_slots(-1) == 0 and B.fastgl_idmap_table_slots(2 ** 30) == 0
    cap = B.fastgl_idmap_table_slots(3_000_000)
    assert cap == 4_500_000                      # 1.5 slots per input ID: never full, whatever repeats
    assert B.fastgl_idmap_workspace_bytes(500_000, 2_500_000) >= 16 * cap + 4 * 3_000_000
    assert B.fastgl_idmap_workspace_bytes(-1, 5) == 0
    f = L.fastgl_idmap
    assert f(FAKE, -1, FAKE, 4, 0, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == B.FASTGL_ERR_INVALID_ARG
    assert f(FAKE, 4, FAKE, 2 ** 30, 0, FAKE, FAKE, FAKE, FAKE, 1 << 40, None) == B.FASTGL_ERR_UNSUPPORTED
    assert f(FAKE, 4, FAKE, 4, 2, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == B.FASTGL_ERR_INVALID_ARG
    assert "mode" in B.fastgl_last_error()
    assert f(None, 4, FAKE, 4, 0, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == B.FASTGL_ERR_INVALID_ARG
    assert f(FAKE, 4, FAKE, 4, 0, FAKE, FAKE, None, FAKE, 1 << 30, None) == B.FASTGL_ERR_INVALID_ARG
    assert f(FAKE, 4, ctypes.c_void_p(0x1004), 4, 0, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == B.FASTGL_ERR_INVALID_ARG
    assert "aligned" in B.fastgl_last_error()
    assert f(FAKE, 4, FAKE, 4, 0, FAKE, FAKE, FAKE, None, 1 << 30, None) == B.FASTGL_ERR_INVALID_ARG
    assert f(FAKE, 4, FAKE, 4, 0, FAKE, FAKE, FAKE, FAKE, 64, None) == B.FASTGL_ERR_WORKSPACE


def test_match_argument_checks_and_host_reorder():
    L = B.lib()
    assert B.fastgl_match_workspace_bytes(1000, 10) >= 16 * 2000          # two slots per ID of the last mini-batch
    assert B.fastgl_match_workspace_bytes(-1, 10) == 0 and B.fastgl_overlap_workspace_bytes(-1) == 0
    assert B.fastgl_overlap_workspace_bytes(1000) >= 16 * 2000 + 4000
    m = L.fastgl_match
    assert m(FAKE, -1, FAKE, 4, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == B.FASTGL_ERR_INVALID_ARG
    assert m(FAKE, 2 ** 30, FAKE, 4, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 40, None) == B.FASTGL_ERR_UNSUPPORTED
    assert m(FAKE, 4, None, 4, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == B.FASTGL_ERR_INVALID_ARG
    assert m(FAKE, 4, FAKE, 4, FAKE, FAKE, FAKE, FAKE, None, 1 << 30, None) == B.FASTGL_ERR_INVALID_ARG
    assert m(FAKE, 4, FAKE, 4, FAKE, FAKE, FAKE, FAKE, FAKE, 64, None) == B.FASTGL_ERR_WORKSPACE
    a = L.fastgl_assemble_rows
    assert a(FAKE, 4, FAKE, 4, FAKE, 4, 0, 0, FAKE, None) == B.FASTGL_ERR_INVALID_ARG
    assert a(FAKE, 4, FAKE, 4, FAKE, 4, 8, 2, FAKE, None) == B.FASTGL_ERR_INVALID_ARG
    assert a(FAKE, 4, FAKE, 4, None, 4, 8, 0, FAKE, None) == B.FASTGL_ERR_INVALID_ARG
    assert a(FAKE, 4, FAKE, 4, FAKE, 0, 8, 0, None, None) == B.FASTGL_OK                    # nothing to do
    off = (ctypes.c_int64 * 3)(0, 5, 3)
    o = L.fastgl_overlap_counts
    assert o(FAKE, off, 2, FAKE, FAKE, FAKE, 1 << 30, None) == B.FASTGL_ERR_INVALID_ARG
    assert "offsets" in B.fastgl_last_error()
    assert o(FAKE, off, 65, FAKE, FAKE, FAKE, 1 << 30, None) == B.FASTGL_ERR_INVALID_ARG
    # Algorithm 1 runs on the host: no GPU needed
    assert B.fastgl_greedy_reorder([], []) == []
    assert B.fastgl_greedy_reorder([[7]], [7]) == [0]
    O = [[9, 5, 4, 0], [5, 9, 0, 1], [4, 0, 9, 8], [0, 1, 8, 9]]
    assert B.fastgl_greedy_reorder(O, [9, 9, 9, 9]) == [0, 1, 3, 2]
    assert B.fastgl_greedy_reorder([[10, 2, 5], [2, 10, 0], [5, 0, 10]], [10, 10, 10]) == [0, 2, 1]
    assert B.fastgl_greedy_reorder([[3, 0, 0], [0, 3, 0], [0, 0, 3]], [3, 3, 3]) == [0, 1, 2]   # ties: smallest index


def test_host_reorder_against_oracle():
    import numpy as np
    import oracle
    rng = np.random.default_rng(5)
    for n in (1, 2, 5, 9, 17):
        sets = [rng.choice(80, size=int(rng.integers(4, 40)), replace=False) for _ in range(n)]
        sizes = [len(s) for s in sets]
        O = oracle.overlap_matrix(sets)
        assert B.fastgl_greedy_reorder(O.tolist(), sizes) == oracle.greedy_reorder(O, sizes).tolist()


def test_edge_argument_checks():
    L = B.lib()
    assert B.fastgl_edge_softmax_long_row() >= 64
    assert B.fastgl_edge_workspace_bytes(10, 1000) >= 4000 and B.fastgl_edge_workspace_bytes(-1, 5) == 0
    g = L.fastgl_edge_weight_grad

    def grad(indptr=FAKE, indices=FAKE, nd=4, ns=4, ne=4, feat=8, mode=0, dt=0, X=FAKE, G=FAKE, plan=None, gw=FAKE,
             ws=FAKE, wsb=1 << 30):
        return g(indptr, indices, nd, ns, ne, feat, mode, dt, X, G, plan, gw, ws, wsb, None)
    assert grad(nd=-1) == B.FASTGL_ERR_INVALID_ARG
    assert grad(feat=0) == B.FASTGL_ERR_INVALID_ARG
    assert grad(mode=3) == B.FASTGL_ERR_INVALID_ARG
    assert grad(X=None) == B.FASTGL_ERR_INVALID_ARG
    assert grad(mode=2) == B.FASTGL_ERR_INVALID_ARG and "plan" in B.fastgl_last_error()
    assert grad(ws=None) == B.FASTGL_ERR_INVALID_ARG
    assert grad(wsb=8) == B.FASTGL_ERR_WORKSPACE
    assert grad(ne=0, indices=None, X=None) == B.FASTGL_OK                    # nothing to do
    f = L.fastgl_edge_softmax_fwd
    assert f(None, 4, 4, FAKE, FAKE, FAKE, 1 << 30, None) == B.FASTGL_ERR_INVALID_ARG
    assert f(FAKE, 4, 4, None, FAKE, FAKE, 1 << 30, None) == B.FASTGL_ERR_INVALID_ARG
    assert f(FAKE, 4, 4, FAKE, FAKE, FAKE, 8, None) == B.FASTGL_ERR_WORKSPACE
    assert f(FAKE, 0, 4, FAKE, FAKE, FAKE, 1 << 30, None) == B.FASTGL_ERR_INVALID_ARG
    b = L.fastgl_edge_softmax_bwd
    assert b(FAKE, 4, 4, FAKE, None, FAKE, FAKE, 1 << 30, None) == B.FASTGL_ERR_INVALID_ARG
    assert b(FAKE, 4, 0, None, None, None, None, 0, None) == B.FASTGL_OK
    s = L.fastgl_edge_score_fwd
    nan = float("nan")
    assert s(FAKE, FAKE, 4, 4, 4, FAKE, FAKE, 0.2, None, None) == B.FASTGL_ERR_INVALID_ARG       # no score array
    assert s(FAKE, FAKE, 4, 4, 4, FAKE, FAKE, nan, FAKE, None) == B.FASTGL_ERR_INVALID_ARG and "slope" in B.fastgl_last_error()
    assert s(FAKE, FAKE, 4, 4, 4, None, FAKE, 0.2, FAKE, None) == B.FASTGL_ERR_INVALID_ARG
    assert s(FAKE, FAKE, 4, -1, 4, FAKE, FAKE, 0.2, FAKE, None) == B.FASTGL_ERR_INVALID_ARG
    assert s(FAKE, None, 4, 4, 0, None, None, 0.2, None, None) == B.FASTGL_OK                     # no edges
    sb = L.fastgl_edge_score_bwd
    assert sb(FAKE, FAKE, 4, 4, 4, FAKE, FAKE, 0.2, None, None, FAKE, None, None) == B.FASTGL_ERR_INVALID_ARG   # grad_score
    assert sb(FAKE, FAKE, 4, 4, 4, FAKE, FAKE, 0.2, FAKE, None, None, FAKE, None) == B.FASTGL_ERR_INVALID_ARG
    assert "FASTGL_PLAN_PERM" in B.fastgl_last_error()                                                 # grad_er needs the plan
    # both gradients asked for, plan missing: refused before the grad_el kernel is enqueued
    assert sb(FAKE, FAKE, 4, 4, 4, FAKE, FAKE, 0.2, FAKE, None, FAKE, FAKE, None) == B.FASTGL_ERR_INVALID_ARG
    assert "FASTGL_PLAN_PERM" in B.fastgl_last_error()
    assert sb(FAKE, FAKE, 4, 4, 4, FAKE, FAKE, 0.2, FAKE, None, None, None, None) == B.FASTGL_OK      # nothing asked for

"""ctypes front end of the CPU oracle (oracle/fastgl_oracle.c, oracle/update_oracle.c,
oracle/idmap_oracle.c, oracle/match_oracle.c, oracle/edge_oracle.c).

TEST INFRASTRUCTURE ONLY.  Only tests/, the smoke check and the benchmark's
cpu_baseline leg may import this package; the product path never does.  It
works on host numpy arrays and imports nothing from the GPU package.

Formulas: paper Section 2.1 Eq. 1 (forward) and Section 4.2 Eq. 5 (backward,
read as the transpose of Eq. 1 applied to the upstream gradient); Section 2.1
Eq. 2 (update phase, read as the GCN dense transform act(H W + b)); Section 2.2 and Section 4.3,
Algorithm 2 (ID map: global IDs to consecutive local IDs); Section 4.1 (Match process, match degree,
Algorithm 1: Greedy Reorder Strategy); Eq. 1 differentiated with respect to the edge weights, and
the softmax over a target node's incoming edges that produces attention weights.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fastgl_oracle.c")
_SRCS = [_SRC, os.path.join(_HERE, "update_oracle.c"), os.path.join(_HERE, "idmap_oracle.c"),
         os.path.join(_HERE, "match_oracle.c"), os.path.join(_HERE, "edge_oracle.c")]
_LIB = os.path.join(_HERE, "libfastgl_oracle.so")

MODES = {"sum": 0, "mean": 1, "gcn": 2}
DTYPES = {"f32": 0, "bf16": 1}


# FASTGL_ORACLE_UBSAN=1 in the environment: the same sources built with the undefined-behaviour
# sanitizer (every finding aborts the process); tests/test_sanitizers.py runs the pin tests on it.
_UBSAN = os.environ.get("FASTGL_ORACLE_UBSAN") == "1"
if _UBSAN:
    _LIB = os.path.join(_HERE, "libfastgl_oracle_ubsan.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (generic x86-64 so the .so runs on any host)."""
    if (force or not os.path.exists(_LIB)
            or os.path.getmtime(_LIB) < max(os.path.getmtime(f) for f in _SRCS)):
        extra = ["-fsanitize=undefined", "-fno-sanitize-recover=all", "-g"] if _UBSAN else []
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", *extra,
               "-Wall", "-Wextra", "-o", _LIB, *_SRCS, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_LIB_TIMED = os.path.join(_HERE, "libfastgl_oracle_timed.so")
TIMED_FLAGS = ["-O3", "-march=native", "-fopenmp"]


def _host_signature() -> str:
    """What -march=native depends on: the CPU model and its feature flags."""
    model = flags = ""
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name") and not model:
                    model = line.split(":", 1)[1].strip()
                elif line.startswith("flags") and not flags:
                    flags = line.split(":", 1)[1].strip()
                if model and flags:
                    break
    except OSError:
        pass
    import hashlib
    return model + " " + hashlib.sha1(flags.encode()).hexdigest()[:12]


def build_timed(force: bool = False) -> str:
    """The same source (fastgl_oracle.c: the parallel variant and the transpose it uses) compiled for
    the benchmark's cpu_baseline leg with TIMED_FLAGS.  -march=native binds the library to the host
    it was compiled on, so it is rebuilt whenever the host differs from the one recorded next to it.
    Parity tests never load this library."""
    stamp = _LIB_TIMED + ".host"
    sig = _host_signature()
    stale = (force or not os.path.exists(_LIB_TIMED) or not os.path.exists(stamp)
             or open(stamp).read() != sig or os.path.getmtime(_LIB_TIMED) < os.path.getmtime(_SRC))
    if stale:
        subprocess.run(["gcc", *TIMED_FLAGS, "-std=c11", "-fPIC", "-shared", "-o", _LIB_TIMED, _SRC, "-lm"], check=True)
        with open(stamp, "w") as f:
            f.write(sig)
    return _LIB_TIMED


def build_sanitize_check() -> str:
    """oracle/sanitize_check.c (the driver of the sanitizer test) as a plain executable, so that the
    build check covers every C file of this folder; tests/test_sanitizers.py builds its own copy with
    the sanitizers on."""
    exe = os.path.join(_HERE, "sanitize_check.bin")
    subprocess.run(["gcc", "-O1", "-std=c11", "-fopenmp", "-Wall", "-Wextra", "-o", exe,
                    os.path.join(_HERE, "sanitize_check.c"), *_SRCS, "-lm"], check=True)
    return exe


_lib_timed = None


def timed_lib():
    global _lib_timed
    if _lib_timed is None:
        L = ctypes.CDLL(build_timed())
        p, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        for name in ("fastgl_oracle_par_aggregate_fwd", "fastgl_oracle_par_aggregate_bwd"):
            getattr(L, name).argtypes = [p, p, p, i64, i64, i64, i64, i32, i32, p, p]
            getattr(L, name).restype = i32
        L.fastgl_oracle_num_threads.restype = i32
        _lib_timed = L
    return _lib_timed


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        p, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        agg = [p, p, p, i64, i64, i64, i64, i32, i32, p, p]
        for name in ("fastgl_oracle_aggregate_fwd", "fastgl_oracle_aggregate_bwd",
                     "fastgl_oracle_par_aggregate_fwd", "fastgl_oracle_par_aggregate_bwd"):
            getattr(L, name).argtypes = agg
            getattr(L, name).restype = i32
        L.fastgl_oracle_degrees.argtypes = [p, p, i64, i64, i64, p, p]
        L.fastgl_oracle_degrees.restype = i32
        L.fastgl_oracle_transpose.argtypes = [p, p, i64, i64, i64, p, p, p]
        L.fastgl_oracle_transpose.restype = i32
        L.fastgl_oracle_long_rows.argtypes = [p, i64, ctypes.c_int32, ctypes.c_int32, p, p]
        L.fastgl_oracle_long_rows.restype = i64
        L.fastgl_oracle_work_split.argtypes = [p, i64, ctypes.c_int32, p]
        L.fastgl_oracle_work_split.restype = i64
        L.fastgl_oracle_gather_rows.argtypes = [p, p, i64, i64, i32, p]
        L.fastgl_oracle_gather_rows.restype = i32
        L.fastgl_oracle_double_to_bf16.argtypes = [ctypes.c_double]
        L.fastgl_oracle_double_to_bf16.restype = ctypes.c_uint16
        L.fastgl_oracle_num_threads.restype = i32
        L.fastgl_oracle_update_fwd.argtypes = [p, p, p, i64, i64, i64, i32, p]
        L.fastgl_oracle_update_fwd.restype = i32
        L.fastgl_oracle_update_bwd.argtypes = [p, p, p, p, i64, i64, i64, i32, p, p, p]
        L.fastgl_oracle_update_bwd.restype = i32
        L.fastgl_oracle_update_fwd_dt.argtypes = [p, p, p, i64, i64, i64, i32, i32, p]
        L.fastgl_oracle_update_fwd_dt.restype = i32
        L.fastgl_oracle_update_bwd_dt.argtypes = [p, p, p, p, i64, i64, i64, i32, i32, p, p, p]
        L.fastgl_oracle_update_bwd_dt.restype = i32
        L.fastgl_oracle_edge_weight_grad.argtypes = [p, p, i64, i64, i64, i32, i32, p, p, p, p]
        L.fastgl_oracle_edge_weight_grad.restype = i32
        L.fastgl_oracle_edge_softmax_fwd.argtypes = [p, i64, p, p]
        L.fastgl_oracle_edge_softmax_fwd.restype = i32
        L.fastgl_oracle_edge_softmax_bwd.argtypes = [p, i64, p, p, p]
        L.fastgl_oracle_edge_softmax_bwd.restype = i32
        L.fastgl_oracle_edge_score_fwd.argtypes = [p, p, i64, i64, p, p, ctypes.c_double, p]
        L.fastgl_oracle_edge_score_fwd.restype = i32
        L.fastgl_oracle_edge_score_bwd.argtypes = [p, p, i64, i64, p, p, ctypes.c_double, p, p, p, p]
        L.fastgl_oracle_edge_score_bwd.restype = i32
        L.fastgl_oracle_match.argtypes = [p, i64, p, i64, p, p, p]
        L.fastgl_oracle_match.restype = i64
        L.fastgl_oracle_overlap.argtypes = [p, i64, p, i64]
        L.fastgl_oracle_overlap.restype = i64
        L.fastgl_oracle_greedy_reorder.argtypes = [p, p, i64, p]
        L.fastgl_oracle_greedy_reorder.restype = i32
        L.fastgl_oracle_assemble.argtypes = [p, p, p, i64, i64, i64, p]
        L.fastgl_oracle_assemble.restype = i32
        L.fastgl_oracle_idmap.argtypes = [p, i64, p, i64, p, p]
        L.fastgl_oracle_idmap.restype = i64
        L.fastgl_oracle_fused_map_seq.argtypes = [p, i64, i64, p, p, p]
        L.fastgl_oracle_fused_map_seq.restype = i64
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _feat_array(a, dtype):
    want = np.float32 if dtype == "f32" else np.uint16
    a = np.ascontiguousarray(a)
    if a.dtype != want:
        raise TypeError(f"{dtype} features must be {want} (bf16 as uint16 bit patterns)")
    return a


def _aggregate(fn, indptr, indices, edge_w, num_src, mode, dtype, inp, out_rows):
    indptr, indices = _i32(indptr), _i32(indices)
    inp = _feat_array(inp, dtype)
    num_dst = indptr.shape[0] - 1
    feat = inp.shape[1]
    w = None if edge_w is None else np.ascontiguousarray(edge_w, dtype=np.float32)
    out = np.empty((out_rows, feat), dtype=inp.dtype)
    rc = fn(_ptr(indptr), _ptr(indices), _ptr(w), num_dst, num_src, indices.shape[0], feat,
            MODES[mode], DTYPES[dtype], _ptr(inp), _ptr(out))
    if rc:
        raise RuntimeError(f"oracle returned {rc}")
    return out


def aggregate_fwd(indptr, indices, edge_w, num_src, mode, dtype, X):
    assert X.shape[0] == num_src
    return _aggregate(lib().fastgl_oracle_aggregate_fwd, indptr, indices, edge_w, num_src,
                      mode, dtype, X, len(indptr) - 1)


def aggregate_bwd(indptr, indices, edge_w, num_src, mode, dtype, G):
    assert G.shape[0] == len(indptr) - 1
    return _aggregate(lib().fastgl_oracle_aggregate_bwd, indptr, indices, edge_w, num_src,
                      mode, dtype, G, num_src)


def par_aggregate_fwd(indptr, indices, edge_w, num_src, mode, dtype, X, timed=False):
    """timed=True: the build with TIMED_FLAGS (what the benchmark times); same source, same result
    up to fp32 contraction."""
    L = timed_lib() if timed else lib()
    return _aggregate(L.fastgl_oracle_par_aggregate_fwd, indptr, indices, edge_w, num_src,
                      mode, dtype, X, len(indptr) - 1)


def par_aggregate_bwd(indptr, indices, edge_w, num_src, mode, dtype, G, timed=False):
    L = timed_lib() if timed else lib()
    return _aggregate(L.fastgl_oracle_par_aggregate_bwd, indptr, indices, edge_w, num_src,
                      mode, dtype, G, num_src)


def degrees(indptr, indices, num_src):
    indptr, indices = _i32(indptr), _i32(indices)
    num_dst = indptr.shape[0] - 1
    din = np.empty(num_dst, np.int32)
    dout = np.empty(num_src, np.int32)
    rc = lib().fastgl_oracle_degrees(_ptr(indptr), _ptr(indices), num_dst, num_src,
                                     indices.shape[0], _ptr(din), _ptr(dout))
    if rc:
        raise ValueError("index out of range")
    return din, dout


def transpose(indptr, indices, num_src):
    indptr, indices = _i32(indptr), _i32(indices)
    num_dst = indptr.shape[0] - 1
    e = indices.shape[0]
    pT = np.empty(num_src + 1, np.int32)
    iT = np.empty(e, np.int32)
    perm = np.empty(e, np.int32)
    rc = lib().fastgl_oracle_transpose(_ptr(indptr), _ptr(indices), num_dst, num_src, e,
                                       _ptr(pT), _ptr(iT), _ptr(perm))
    if rc:
        raise RuntimeError(f"oracle returned {rc}")
    return pT, iT, perm


def long_rows(rowptr, threshold, chunk):
    rowptr = _i32(rowptr)
    n = rowptr.shape[0] - 1
    rows = np.empty(n + 1, np.int32)
    cptr = np.empty(n + 2, np.int32)
    k = lib().fastgl_oracle_long_rows(_ptr(rowptr), n, threshold, chunk, _ptr(rows), _ptr(cptr))
    return rows[:k].copy(), cptr[:k + 1].copy()


def work_split(rowptr, work):
    rowptr = _i32(rowptr)
    n = rowptr.shape[0] - 1
    out = np.empty((int(rowptr[-1]) + n) // work + 3, np.int32)
    g = lib().fastgl_oracle_work_split(_ptr(rowptr), n, work, _ptr(out))
    return out[:g + 1].copy()


def gather_rows(table, ids, dtype):
    table = _feat_array(table, dtype)
    ids = np.ascontiguousarray(ids, dtype=np.int64)
    out = np.empty((ids.shape[0], table.shape[1]), dtype=table.dtype)
    lib().fastgl_oracle_gather_rows(_ptr(table), _ptr(ids), ids.shape[0], table.shape[1],
                                    DTYPES[dtype], _ptr(out))
    return out


def double_to_bf16(x: float) -> int:
    return int(lib().fastgl_oracle_double_to_bf16(float(x)))


def num_threads() -> int:
    return int(lib().fastgl_oracle_num_threads())


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def update_fwd(H, W, b, relu):
    """Y = act(H W + b); H [M,K], W [K,N], b [N] or None (Section 2.1, Eq. 2)."""
    H, W = _f32(H), _f32(W)
    b = None if b is None else _f32(b)
    M, K = H.shape
    assert W.shape[0] == K and (b is None or b.shape == (W.shape[1],))
    Y = np.empty((M, W.shape[1]), np.float32)
    rc = lib().fastgl_oracle_update_fwd(_ptr(H), _ptr(W), _ptr(b), M, K, W.shape[1], int(bool(relu)), _ptr(Y))
    if rc:
        raise RuntimeError(f"oracle returned {rc}")
    return Y


def update_bwd(H, W, Y, dY, relu, want=("dH", "dW", "db")):
    """Gradients of Eq. 2's dense transform; returns (dH, dW, db), None for parts not wanted.
    Y is the forward output and gates dY where relu is set."""
    H, W, dY = _f32(H), _f32(W), _f32(dY)
    Y = None if Y is None else _f32(Y)
    assert not relu or Y is not None
    M, K = H.shape
    N = W.shape[1]
    assert dY.shape == (M, N) and W.shape[0] == K
    dH = np.empty((M, K), np.float32) if "dH" in want else None
    dW = np.empty((K, N), np.float32) if "dW" in want else None
    db = np.empty(N, np.float32) if "db" in want else None
    rc = lib().fastgl_oracle_update_bwd(_ptr(H), _ptr(W), _ptr(Y), _ptr(dY), M, K, N, int(bool(relu)),
                                        _ptr(dH), _ptr(dW), _ptr(db))
    if rc:
        raise RuntimeError(f"oracle returned {rc}")
    return dH, dW, db


def idmap(dst_gid, nbr_gid):
    """ID map of one sampled hop (Section 2.2; Section 4.3): destinations keep 0..n_dst-1, every
    other node is numbered by first appearance in the neighbour list.
    Returns (local_nbr int32[n_nbr], unique_gid int64[U])."""
    dst = np.ascontiguousarray(dst_gid, dtype=np.int64)
    nbr = np.ascontiguousarray(nbr_gid, dtype=np.int64)
    local = np.empty(nbr.shape[0], np.int32)
    uniq = np.empty(dst.shape[0] + nbr.shape[0], np.int64)
    U = lib().fastgl_oracle_idmap(_ptr(dst), dst.shape[0], _ptr(nbr), nbr.shape[0], _ptr(local), _ptr(uniq))
    if U == -2:
        raise ValueError("destination IDs repeat")
    if U < 0:
        raise RuntimeError(f"oracle returned {U}")
    return local, uniq[:U].copy()


def fused_map_sequential(ids, table_size):
    """Algorithm 2 run by one thread with HashFunction = id mod table_size.
    Returns (key int64[table_size], value int64[table_size], local int64[n], LocalID)."""
    ids = np.ascontiguousarray(ids, dtype=np.int64)
    key = np.empty(table_size, np.int64)
    value = np.empty(table_size, np.int64)
    local = np.empty(ids.shape[0], np.int64)
    U = lib().fastgl_oracle_fused_map_seq(_ptr(ids), ids.shape[0], table_size, _ptr(key), _ptr(value), _ptr(local))
    if U < 0:
        raise RuntimeError("hash table full")
    return key, value, local, int(U)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def match(prev_gid, new_gid):
    """Match process (Section 4.1): returns (match_row int32[n_new] = row in the last mini-batch or
    -1, load_pos int32[n_load] ascending, load_gid int64[n_load])."""
    prev, new = _i64(prev_gid), _i64(new_gid)
    mrow = np.empty(new.shape[0], np.int32)
    lpos = np.empty(new.shape[0], np.int32)
    lgid = np.empty(new.shape[0], np.int64)
    k = lib().fastgl_oracle_match(_ptr(prev), prev.shape[0], _ptr(new), new.shape[0], _ptr(mrow), _ptr(lpos),
                                  _ptr(lgid))
    if k == -2:
        raise ValueError("IDs of the last mini-batch repeat")
    if k < 0:
        raise RuntimeError(f"oracle returned {k}")
    return mrow, lpos[:k].copy(), lgid[:k].copy()


def overlap(a, b) -> int:
    a, b = _i64(a), _i64(b)
    return int(lib().fastgl_oracle_overlap(_ptr(a), a.shape[0], _ptr(b), b.shape[0]))


def match_degree(a, b) -> float:
    """M_ij = N_o / min(N_i, N_j) (Section 4.1)."""
    return overlap(a, b) / min(len(a), len(b))


def overlap_matrix(batches):
    n = len(batches)
    O = np.zeros((n, n), np.int64)
    for i in range(n):
        for j in range(n):
            O[i, j] = len(batches[i]) if i == j else overlap(batches[i], batches[j])
    return O


def greedy_reorder(overlap_counts, sizes):
    """Algorithm 1: returns the ReorderedList as 0-based mini-batch indices."""
    O, sz = _i64(overlap_counts), _i64(sizes)
    n = sz.shape[0]
    assert O.shape == (n, n)
    order = np.empty(n, np.int32)
    if lib().fastgl_oracle_greedy_reorder(_ptr(O), _ptr(sz), n, _ptr(order)):
        raise RuntimeError("oracle failed")
    return order


def assemble(X_prev, X_load, match_row):
    X_prev, X_load = np.ascontiguousarray(X_prev), np.ascontiguousarray(X_load)
    mrow = _i32(match_row)
    assert X_prev.dtype == X_load.dtype and X_prev.shape[1:] == X_load.shape[1:]
    feat = X_prev.shape[1]
    out = np.empty((mrow.shape[0], feat), X_prev.dtype)
    assert int((mrow < 0).sum()) == X_load.shape[0]
    if lib().fastgl_oracle_assemble(_ptr(X_prev), _ptr(X_load), _ptr(mrow), mrow.shape[0], feat,
                                    X_prev.dtype.itemsize, _ptr(out)):
        raise RuntimeError("oracle failed")
    return out


def edge_weight_grad(indptr, indices, num_src, mode, dtype, X, G):
    """dL/dw_e = c_u s_v <G[u], X[v]> for every edge (Eq. 1 differentiated by its weights)."""
    indptr, indices = _i32(indptr), _i32(indices)
    X, G = _feat_array(X, dtype), _feat_array(G, dtype)
    num_dst = indptr.shape[0] - 1
    assert X.shape[0] == num_src and G.shape == (num_dst, X.shape[1])
    gw = np.empty(indices.shape[0], np.float32)
    scratch = np.empty(max(num_src, 1), np.int32)
    rc = lib().fastgl_oracle_edge_weight_grad(_ptr(indptr), _ptr(indices), num_dst, num_src, X.shape[1],
                                              MODES[mode], DTYPES[dtype], _ptr(X), _ptr(G), _ptr(scratch), _ptr(gw))
    if rc:
        raise RuntimeError(f"oracle returned {rc}")
    return gw


def edge_softmax_fwd(indptr, score):
    indptr, score = _i32(indptr), _f32(score)
    assert score.shape[0] == indptr[-1]
    alpha = np.zeros_like(score)
    if lib().fastgl_oracle_edge_softmax_fwd(_ptr(indptr), indptr.shape[0] - 1, _ptr(score), _ptr(alpha)):
        raise RuntimeError("oracle failed")
    return alpha


def edge_softmax_bwd(indptr, alpha, grad_alpha):
    indptr, alpha, grad_alpha = _i32(indptr), _f32(alpha), _f32(grad_alpha)
    out = np.zeros_like(alpha)
    if lib().fastgl_oracle_edge_softmax_bwd(_ptr(indptr), indptr.shape[0] - 1, _ptr(alpha), _ptr(grad_alpha),
                                            _ptr(out)):
        raise RuntimeError("oracle failed")
    return out


def edge_score_fwd(indptr, indices, el, er, slope):
    """Attention logits of a GAT head: LeakyReLU(el[u] + er[v]) for every edge (u, v).  The slope is an
    fp32 parameter of the layer, like el and er: it is rounded to fp32 before use."""
    slope = float(np.float32(slope))
    indptr, indices, el, er = _i32(indptr), _i32(indices), _f32(el), _f32(er)
    assert el.shape[0] == indptr.shape[0] - 1
    score = np.zeros(indices.shape[0], np.float32)
    if lib().fastgl_oracle_edge_score_fwd(_ptr(indptr), _ptr(indices), el.shape[0], er.shape[0], _ptr(el), _ptr(er), float(slope), _ptr(score)):
        raise RuntimeError("oracle failed")
    return score


def edge_score_bwd(indptr, indices, el, er, slope, grad_score):
    """(grad_el, grad_er) of the attention logits (slope rounded to fp32 as in the forward pass)."""
    slope = float(np.float32(slope))
    indptr, indices, el, er, grad_score = _i32(indptr), _i32(indices), _f32(el), _f32(er), _f32(grad_score)
    g_el, g_er = np.zeros(el.shape[0], np.float32), np.zeros(er.shape[0], np.float32)
    acc = np.zeros(max(er.shape[0], 1), np.float64)
    if lib().fastgl_oracle_edge_score_bwd(_ptr(indptr), _ptr(indices), el.shape[0], er.shape[0], _ptr(el), _ptr(er),
                                          float(slope), _ptr(grad_score), _ptr(acc), _ptr(g_el), _ptr(g_er)):
        raise RuntimeError("oracle failed")
    return g_el, g_er


def update_fwd_bf16(H, W, b, relu):
    """Eq. 2 with bf16 storage: H, W and the result are bf16 bit patterns (uint16), the bias fp32."""
    H, W = _feat_array(H, "bf16"), _feat_array(W, "bf16")
    b = None if b is None else _f32(b)
    M, K = H.shape
    assert W.shape[0] == K
    Y = np.empty((M, W.shape[1]), np.uint16)
    if lib().fastgl_oracle_update_fwd_dt(_ptr(H), _ptr(W), _ptr(b), M, K, W.shape[1], int(bool(relu)), 1, _ptr(Y)):
        raise RuntimeError("oracle failed")
    return Y


def update_bwd_bf16(H, W, Y, dY, relu, want=("dH", "dW", "db")):
    """Gradients with bf16 storage: H, W, Y, dY and dH are bf16 bit patterns, dW and db fp32."""
    H, W, dY = _feat_array(H, "bf16"), _feat_array(W, "bf16"), _feat_array(dY, "bf16")
    Y = None if Y is None else _feat_array(Y, "bf16")
    assert not relu or Y is not None
    M, K = H.shape
    N = W.shape[1]
    dH = np.empty((M, K), np.uint16) if "dH" in want else None
    dW = np.empty((K, N), np.float32) if "dW" in want else None
    db = np.empty(N, np.float32) if "db" in want else None
    if lib().fastgl_oracle_update_bwd_dt(_ptr(H), _ptr(W), _ptr(Y), _ptr(dY), M, K, N, int(bool(relu)), 1,
                                         _ptr(dH), _ptr(dW), _ptr(db)):
        raise RuntimeError("oracle failed")
    return dH, dW, db

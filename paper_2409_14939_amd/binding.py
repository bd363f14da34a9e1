"""ctypes binding of libfastgl_agg.so - same names as the C ABI, argument
marshalling only.  PyTorch supplies device memory and the stream handle; every
step of the computation runs in the library's kernels.  There is no fallback:
if the library is missing or an entry point fails, this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfastgl_agg.so")

FASTGL_OK = 0
FASTGL_ERR_INVALID_ARG, FASTGL_ERR_UNSUPPORTED, FASTGL_ERR_WORKSPACE, FASTGL_ERR_HIP = 1, 2, 3, 4
MODES = {"sum": 0, "mean": 1, "gcn": 2}
DTYPES = {"f32": 0, "bf16": 1}
PLAN_FWD, PLAN_BWD, PLAN_ALL, PLAN_SRC_DEG, PLAN_PERM, PLAN_SHORT_DST_ROWS = 1, 2, 3, 4, 8, 16

EXPORTS = [
    "fastgl_block_aggregate_fwd", "fastgl_block_aggregate_bwd", "fastgl_block_aggregate_fwd_static",
    "fastgl_block_plan_bytes",
    "fastgl_block_plan_create", "fastgl_block_plan_create_many", "fastgl_block_plan_export", "fastgl_block_plan_destroy",
    "fastgl_block_workspace_bytes", "fastgl_long_row_threshold", "fastgl_long_row_chunk", "fastgl_work_per_group",
    "fastgl_gather_rows", "fastgl_block_validate", "fastgl_last_error",
    "fastgl_update_fwd", "fastgl_update_bwd", "fastgl_update_bwd_workspace_bytes", "fastgl_update_slab_rows",
    "fastgl_update_fwd_bf16", "fastgl_update_bwd_bf16", "fastgl_layer_fwd", "fastgl_layer_fwd_fuses",
    "fastgl_idmap", "fastgl_idmap_table_slots", "fastgl_idmap_workspace_bytes",
    "fastgl_match", "fastgl_match_workspace_bytes", "fastgl_assemble_rows", "fastgl_overlap_counts",
    "fastgl_overlap_workspace_bytes", "fastgl_greedy_reorder",
    "fastgl_edge_workspace_bytes", "fastgl_edge_weight_grad", "fastgl_edge_softmax_fwd", "fastgl_edge_softmax_bwd",
    "fastgl_edge_softmax_long_row", "fastgl_edge_score_fwd", "fastgl_edge_score_bwd",
]
MAX_REORDER_BATCHES = 64
IDMAP_MODES = {"ordered": 0, "fused": 1}


class FastglError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"fastgl status {status}: {msg}")
        self.status = status


class BlockDesc(ctypes.Structure):
    _fields_ = [("indptr", ctypes.c_void_p), ("indices", ctypes.c_void_p), ("num_dst", ctypes.c_int64),
                ("num_src", ctypes.c_int64), ("num_edges", ctypes.c_int64), ("parts", ctypes.c_int),
                ("plan_mem", ctypes.c_void_p), ("plan_bytes", ctypes.c_size_t)]


class PlanView(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in (
        "din", "dout", "indptr_T", "indices_T", "perm", "dst_inv", "dst_rsqrt", "src_rsqrt",
        "long_dst", "chunk_ptr_dst", "long_src", "chunk_ptr_src", "counters", "split_dst", "split_src")]


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = ctypes.CDLL(LIB_PATH)
        p, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
        agg = [p, p, p, i64, i64, i64, i64, i32, i32, p, p, p, p, sz, p]
        L.fastgl_block_aggregate_fwd.argtypes = agg
        L.fastgl_block_aggregate_bwd.argtypes = agg
        L.fastgl_block_aggregate_fwd_static.argtypes = [p, p, p, i64, i64, i64, i64, i32, i32, p, p, p]
        L.fastgl_block_plan_bytes.argtypes = [i64, i64, i64]
        L.fastgl_block_plan_bytes.restype = sz
        L.fastgl_block_plan_create.argtypes = [p, p, i64, i64, i64, i32, p, sz, p, ctypes.POINTER(p)]
        L.fastgl_block_plan_create_many.argtypes = [i32, ctypes.POINTER(BlockDesc), p, ctypes.POINTER(p)]
        L.fastgl_block_plan_export.argtypes = [p, ctypes.POINTER(PlanView)]
        L.fastgl_block_plan_destroy.argtypes = [p]
        L.fastgl_block_plan_destroy.restype = None
        L.fastgl_block_workspace_bytes.argtypes = [i64, i64, i64, i64, i32]
        L.fastgl_block_workspace_bytes.restype = sz
        L.fastgl_long_row_threshold.restype = ctypes.c_int32
        L.fastgl_long_row_chunk.restype = ctypes.c_int32
        L.fastgl_work_per_group.restype = ctypes.c_int32
        L.fastgl_gather_rows.argtypes = [p, i64, p, i64, i64, i32, p, p]
        L.fastgl_block_validate.argtypes = [p, p, i64, i64, i64, p, ctypes.POINTER(i64), p]
        L.fastgl_last_error.restype = ctypes.c_char_p
        L.fastgl_update_fwd.argtypes = [p, p, p, i64, i64, i64, i32, p, p]
        L.fastgl_update_fwd_bf16.argtypes = L.fastgl_update_fwd.argtypes
        L.fastgl_update_bwd_workspace_bytes.argtypes = [i64, i64, i64]
        L.fastgl_update_bwd_workspace_bytes.restype = sz
        L.fastgl_update_bwd.argtypes = [p, p, p, p, i64, i64, i64, i32, p, p, p, p, sz, p]
        L.fastgl_match_workspace_bytes.argtypes = [i64, i64]
        L.fastgl_match_workspace_bytes.restype = sz
        L.fastgl_match.argtypes = [p, i64, p, i64, p, p, p, p, p, sz, p]
        L.fastgl_assemble_rows.argtypes = [p, i64, p, i64, p, i64, i64, i32, p, p]
        L.fastgl_overlap_workspace_bytes.argtypes = [i64]
        L.fastgl_overlap_workspace_bytes.restype = sz
        L.fastgl_overlap_counts.argtypes = [p, ctypes.POINTER(i64), i32, p, p, p, sz, p]
        L.fastgl_greedy_reorder.argtypes = [ctypes.POINTER(i64), ctypes.POINTER(i64), i64,
                                            ctypes.POINTER(ctypes.c_int32)]
        L.fastgl_edge_workspace_bytes.argtypes = [i64, i64]
        L.fastgl_edge_workspace_bytes.restype = sz
        L.fastgl_edge_weight_grad.argtypes = [p, p, i64, i64, i64, i64, i32, i32, p, p, p, p, p, sz, p]
        L.fastgl_edge_softmax_fwd.argtypes = [p, i64, i64, p, p, p, sz, p]
        L.fastgl_edge_softmax_bwd.argtypes = [p, i64, i64, p, p, p, p, sz, p]
        L.fastgl_edge_softmax_long_row.restype = ctypes.c_int32
        L.fastgl_edge_score_fwd.argtypes = [p, p, i64, i64, i64, p, p, ctypes.c_float, p, p]
        L.fastgl_edge_score_bwd.argtypes = [p, p, i64, i64, i64, p, p, ctypes.c_float, p, p, p, p, p]
        L.fastgl_idmap_table_slots.argtypes = [i64]
        L.fastgl_idmap_table_slots.restype = i64
        L.fastgl_idmap_workspace_bytes.argtypes = [i64, i64]
        L.fastgl_idmap_workspace_bytes.restype = sz
        L.fastgl_idmap.argtypes = [p, i64, p, i64, i32, p, p, p, p, sz, p]
        L.fastgl_update_bwd_bf16.argtypes = L.fastgl_update_bwd.argtypes
        L.fastgl_layer_fwd.argtypes = [p, p, p, i64, i64, i64, i64, i32, i32, p, p, p, i64, i32, p, p, p, p, sz, p]
        L.fastgl_layer_fwd_fuses.argtypes = [i64, i64, i32]
        L.fastgl_update_slab_rows.argtypes = [i64, i64, i64]
        L.fastgl_update_slab_rows.restype = ctypes.c_int32
        _lib = L
    return _lib


def fastgl_last_error() -> str:
    return lib().fastgl_last_error().decode()


def _check(status: int) -> None:
    if status != FASTGL_OK:
        raise FastglError(status, fastgl_last_error())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous device tensor of {dtype}")
    return t


def _feat_dtype(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return DTYPES["f32"]
    if t.dtype == torch.bfloat16:
        return DTYPES["bf16"]
    raise TypeError("features must be float32 or bfloat16")


def fastgl_long_row_threshold() -> int:
    return int(lib().fastgl_long_row_threshold())


def fastgl_long_row_chunk() -> int:
    return int(lib().fastgl_long_row_chunk())


def fastgl_work_per_group() -> int:
    return int(lib().fastgl_work_per_group())


def fastgl_block_plan_bytes(num_dst: int, num_src: int, num_edges: int) -> int:
    return int(lib().fastgl_block_plan_bytes(num_dst, num_src, num_edges))


def fastgl_block_workspace_bytes(num_dst: int, num_src: int, num_edges: int, feat: int, dtype: str) -> int:
    return int(lib().fastgl_block_workspace_bytes(num_dst, num_src, num_edges, feat, DTYPES[dtype]))


class Plan:
    """Owner of one fastgl_plan handle and of the device buffer behind it."""

    def __init__(self, handle, mem, indptr, indices, num_src):
        self.handle, self.mem = handle, mem
        self.indptr, self.indices, self.num_src = indptr, indices, num_src

    def export(self) -> PlanView:
        v = PlanView()
        _check(lib().fastgl_block_plan_export(self.handle, ctypes.byref(v)))
        return v

    def destroy(self) -> None:
        if self.handle is not None and _lib is not None:      # _lib is gone while the interpreter shuts down
            _lib.fastgl_block_plan_destroy(self.handle)
        self.handle = None

    def __del__(self):
        self.destroy()


def fastgl_block_plan_create(indptr: torch.Tensor, indices: torch.Tensor, num_src: int,
                             parts: int = PLAN_ALL, plan_mem: Optional[torch.Tensor] = None) -> Plan:
    _dev(indptr, torch.int32, "indptr")
    _dev(indices, torch.int32, "indices")
    num_dst, num_edges = indptr.numel() - 1, indices.numel()
    if plan_mem is None:
        nbytes = fastgl_block_plan_bytes(num_dst, num_src, num_edges)
        plan_mem = torch.empty(nbytes, dtype=torch.uint8, device=indptr.device)
    out = ctypes.c_void_p()
    _check(lib().fastgl_block_plan_create(_ptr(indptr), _ptr(indices), num_dst, num_src, num_edges, parts,
                                          _ptr(plan_mem), plan_mem.numel(), _stream(), ctypes.byref(out)))
    return Plan(out, plan_mem, indptr, indices, num_src)


def fastgl_block_plan_create_many(blocks, parts: int = PLAN_ALL, plan_mems=None):
    """blocks: list of (indptr, indices, num_src); returns one Plan per block, built together."""
    n = len(blocks)
    descs = (BlockDesc * n)()
    mems = []
    for i, (indptr, indices, num_src) in enumerate(blocks):
        _dev(indptr, torch.int32, "indptr")
        _dev(indices, torch.int32, "indices")
        num_dst, num_edges = indptr.numel() - 1, indices.numel()
        mem = plan_mems[i] if plan_mems is not None else torch.empty(
            fastgl_block_plan_bytes(num_dst, num_src, num_edges), dtype=torch.uint8, device=indptr.device)
        mems.append(mem)
        descs[i] = BlockDesc(indptr.data_ptr(), indices.data_ptr(), num_dst, num_src, num_edges, parts,
                             mem.data_ptr(), mem.numel())
    out = (ctypes.c_void_p * n)()
    _check(lib().fastgl_block_plan_create_many(n, descs, _stream(), out))
    return [Plan(ctypes.c_void_p(out[i]), mems[i], blocks[i][0], blocks[i][1], blocks[i][2]) for i in range(n)]


def _aggregate(fn, indptr, indices, edge_w, num_src, mode, inp, out, plan, workspace):
    _dev(indptr, torch.int32, "indptr")
    _dev(indices, torch.int32, "indices")
    if edge_w is not None:
        _dev(edge_w, torch.float32, "edge_w")
    dt = _feat_dtype(inp)
    _dev(inp, inp.dtype, "input features")
    _dev(out, inp.dtype, "output features")
    num_dst, num_edges, feat = indptr.numel() - 1, indices.numel(), inp.shape[1]
    if workspace is None:
        nbytes = int(lib().fastgl_block_workspace_bytes(num_dst, num_src, num_edges, feat, dt))
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=inp.device)
    _check(fn(_ptr(indptr), _ptr(indices), _ptr(edge_w), num_dst, num_src, num_edges, feat, MODES[mode], dt,
              _ptr(inp), _ptr(out), plan.handle if plan is not None else None, _ptr(workspace),
              workspace.numel(), _stream()))
    return out


def fastgl_block_aggregate_fwd(indptr, indices, edge_w, num_src: int, mode: str, X: torch.Tensor,
                               out: Optional[torch.Tensor] = None, plan: Optional[Plan] = None,
                               workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    if X.shape[0] != num_src:
        raise ValueError("X must have num_src rows")
    if out is None:
        out = torch.empty((indptr.numel() - 1, X.shape[1]), dtype=X.dtype, device=X.device)
    elif out.shape != (indptr.numel() - 1, X.shape[1]):
        raise ValueError("out must be [num_dst, feat]")
    return _aggregate(lib().fastgl_block_aggregate_fwd, indptr, indices, edge_w, num_src, mode, X, out,
                      plan, workspace)


STATIC_SCRATCH_BYTES = 64 << 20


def fastgl_block_aggregate_fwd_static(indptr, indices, edge_w, num_src: int, mode: str, X: torch.Tensor,
                                      out: torch.Tensor) -> torch.Tensor:
    """The forward aggregation on the library's static scratch array: no plan, no workspace, and this
    wrapper allocates nothing either (the caller passes `out`)."""
    _dev(indptr, torch.int32, "indptr")
    _dev(indices, torch.int32, "indices")
    if edge_w is not None:
        _dev(edge_w, torch.float32, "edge_w")
    dt = _feat_dtype(X)
    _dev(X, X.dtype, "X")
    _dev(out, X.dtype, "out")
    num_dst, num_edges, feat = indptr.numel() - 1, indices.numel(), X.shape[1]
    if X.shape[0] != num_src or out.shape != (num_dst, feat):
        raise ValueError("X must be [num_src, feat] and out [num_dst, feat]")
    _check(lib().fastgl_block_aggregate_fwd_static(_ptr(indptr), _ptr(indices), _ptr(edge_w), num_dst, num_src,
                                                   num_edges, feat, MODES[mode], dt, _ptr(X), _ptr(out), _stream()))
    return out


def fastgl_block_aggregate_bwd(indptr, indices, edge_w, num_src: int, mode: str, grad_out: torch.Tensor,
                               grad_X: Optional[torch.Tensor] = None, plan: Optional[Plan] = None,
                               workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    if grad_out.shape[0] != indptr.numel() - 1:
        raise ValueError("grad_out must have num_dst rows")
    if grad_X is None:
        grad_X = torch.empty((num_src, grad_out.shape[1]), dtype=grad_out.dtype, device=grad_out.device)
    elif grad_X.shape != (num_src, grad_out.shape[1]):
        raise ValueError("grad_X must be [num_src, feat]")
    return _aggregate(lib().fastgl_block_aggregate_bwd, indptr, indices, edge_w, num_src, mode, grad_out,
                      grad_X, plan, workspace)


def fastgl_gather_rows(table: torch.Tensor, ids: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    dt = _feat_dtype(table)
    _dev(table, table.dtype, "table")
    _dev(ids, torch.int64, "ids")
    if out is None:
        out = torch.empty((ids.numel(), table.shape[1]), dtype=table.dtype, device=table.device)
    _dev(out, table.dtype, "out")
    _check(lib().fastgl_gather_rows(_ptr(table), table.shape[0], _ptr(ids), ids.numel(), table.shape[1], dt,
                                    _ptr(out), _stream()))
    return out


def fastgl_block_validate(indptr: torch.Tensor, indices: torch.Tensor, num_src: int) -> int:
    _dev(indptr, torch.int32, "indptr")
    _dev(indices, torch.int32, "indices")
    scratch = torch.empty(2, dtype=torch.int64, device=indptr.device)
    n = ctypes.c_int64(-1)
    _check(lib().fastgl_block_validate(_ptr(indptr), _ptr(indices), indptr.numel() - 1, num_src,
                                       indices.numel(), _ptr(scratch), ctypes.byref(n), _stream()))
    return int(n.value)


def fastgl_update_slab_rows(M: int, K: int, N: int) -> int:
    return int(lib().fastgl_update_slab_rows(M, K, N))


def fastgl_update_bwd_workspace_bytes(M: int, K: int, N: int) -> int:
    return int(lib().fastgl_update_bwd_workspace_bytes(M, K, N))


def fastgl_update_fwd(H: torch.Tensor, W: torch.Tensor, bias: Optional[torch.Tensor], relu: bool,
                      Y: Optional[torch.Tensor] = None) -> torch.Tensor:
    """H, W (and Y) float32, or all bfloat16 (the bias stays float32)."""
    dt = H.dtype
    _feat_dtype(H)
    _dev(H, dt, "H")
    _dev(W, dt, "W")
    (M, K), N = H.shape, W.shape[1]
    if W.shape[0] != K or (bias is not None and bias.shape != (N,)):
        raise ValueError("W must be [K,N] and bias [N]")
    if bias is not None:
        _dev(bias, torch.float32, "bias")
    if Y is None:
        Y = torch.empty((M, N), dtype=dt, device=H.device)
    elif Y.shape != (M, N):
        raise ValueError("Y must be [M,N]")
    _dev(Y, dt, "Y")
    fn = lib().fastgl_update_fwd if dt == torch.float32 else lib().fastgl_update_fwd_bf16
    _check(fn(_ptr(H), _ptr(W), _ptr(bias), M, K, N, int(bool(relu)), _ptr(Y), _stream()))
    return Y


def fastgl_layer_fwd_fuses(K: int, N: int, dtype: str) -> bool:
    return bool(lib().fastgl_layer_fwd_fuses(K, N, DTYPES[dtype]))


def fastgl_layer_fwd(indptr, indices, edge_w, num_src: int, mode: str, X: torch.Tensor, W: torch.Tensor,
                     bias: Optional[torch.Tensor], relu: bool, H: Optional[torch.Tensor] = None,
                     Y: Optional[torch.Tensor] = None, want_H: bool = True, plan: Optional[Plan] = None,
                     workspace: Optional[torch.Tensor] = None):
    """Aggregation + update of one layer in one call; returns (H, Y).  want_H=False (and H None) leaves the
    aggregated rows unwritten, which only shapes that fuse allow."""
    _dev(indptr, torch.int32, "indptr")
    _dev(indices, torch.int32, "indices")
    if edge_w is not None:
        _dev(edge_w, torch.float32, "edge_w")
    dt = _feat_dtype(X)
    _dev(X, X.dtype, "X")
    _dev(W, X.dtype, "W")
    num_dst, num_edges, K, N = indptr.numel() - 1, indices.numel(), X.shape[1], W.shape[1]
    if X.shape[0] != num_src or W.shape[0] != K or (bias is not None and bias.shape != (N,)):
        raise ValueError("X must be [num_src,K], W [K,N], bias [N]")
    if bias is not None:
        _dev(bias, torch.float32, "bias")
    if H is None and want_H:
        H = torch.empty((num_dst, K), dtype=X.dtype, device=X.device)
    if Y is None:
        Y = torch.empty((num_dst, N), dtype=X.dtype, device=X.device)
    if H is not None:
        _dev(H, X.dtype, "H")
    _dev(Y, X.dtype, "Y")
    if workspace is None:
        nbytes = int(lib().fastgl_block_workspace_bytes(num_dst, num_src, num_edges, K, dt))
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=X.device)
    _check(lib().fastgl_layer_fwd(_ptr(indptr), _ptr(indices), _ptr(edge_w), num_dst, num_src, num_edges, K,
                                  MODES[mode], dt, _ptr(X), _ptr(W), _ptr(bias), N, int(bool(relu)), _ptr(H), _ptr(Y),
                                  plan.handle if plan is not None else None, _ptr(workspace), workspace.numel(),
                                  _stream()))
    return H, Y


def fastgl_update_bwd(H: torch.Tensor, W: torch.Tensor, Y: Optional[torch.Tensor], dY: torch.Tensor, relu: bool,
                      want=("dH", "dW", "db"), dH=None, dW=None, db=None,
                      workspace: Optional[torch.Tensor] = None):
    """Returns (dH, dW, db); parts not named in `want` (and not passed in) are None.  H, W, Y, dY, dH
    float32, or all bfloat16; dW and db are float32 either way."""
    dt = H.dtype
    _feat_dtype(H)
    _dev(H, dt, "H")
    _dev(W, dt, "W")
    _dev(dY, dt, "dY")
    if Y is not None:
        _dev(Y, dt, "Y")
    (M, K), N = H.shape, W.shape[1]
    if W.shape[0] != K or dY.shape != (M, N) or (Y is not None and Y.shape != (M, N)):
        raise ValueError("shapes must be H [M,K], W [K,N], Y and dY [M,N]")
    if dH is None and "dH" in want:
        dH = torch.empty((M, K), dtype=dt, device=H.device)
    if dW is None and "dW" in want:
        dW = torch.empty((K, N), dtype=torch.float32, device=H.device)
    if db is None and "db" in want:
        db = torch.empty((N,), dtype=torch.float32, device=H.device)
    for t, shape, name in ((dH, (M, K), "dH"), (dW, (K, N), "dW"), (db, (N,), "db")):
        if t is not None:
            _dev(t, dt if name == "dH" else torch.float32, name)
            if tuple(t.shape) != shape:
                raise ValueError(f"{name} must have shape {shape}")
    if workspace is None:
        workspace = torch.empty(max(fastgl_update_bwd_workspace_bytes(M, K, N), 256), dtype=torch.uint8,
                                device=H.device)
    fn = lib().fastgl_update_bwd if dt == torch.float32 else lib().fastgl_update_bwd_bf16
    _check(fn(_ptr(H), _ptr(W), _ptr(Y), _ptr(dY), M, K, N, int(bool(relu)), _ptr(dH), _ptr(dW), _ptr(db),
              _ptr(workspace), workspace.numel(), _stream()))
    return dH, dW, db


def fastgl_idmap_table_slots(n_ids: int) -> int:
    return int(lib().fastgl_idmap_table_slots(n_ids))


def fastgl_idmap_workspace_bytes(n_dst: int, n_nbr: int) -> int:
    return int(lib().fastgl_idmap_workspace_bytes(n_dst, n_nbr))


def fastgl_idmap(dst_gid: torch.Tensor, nbr_gid: torch.Tensor, mode: str = "ordered",
                 local_nbr: Optional[torch.Tensor] = None, unique_gid: Optional[torch.Tensor] = None,
                 result: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None):
    """Returns (local_nbr int32[n_nbr], unique_gid int64[n_dst+n_nbr], result int32[2]) - all on the
    device, nothing is synchronised: result[0] = number of distinct IDs, result[1] = violations."""
    _dev(dst_gid, torch.int64, "dst_gid")
    _dev(nbr_gid, torch.int64, "nbr_gid")
    n_dst, n_nbr = dst_gid.numel(), nbr_gid.numel()
    dev = dst_gid.device
    if local_nbr is None:
        local_nbr = torch.empty(n_nbr, dtype=torch.int32, device=dev)
    if unique_gid is None:
        unique_gid = torch.empty(max(n_dst + n_nbr, 1), dtype=torch.int64, device=dev)
    if result is None:
        result = torch.empty(2, dtype=torch.int32, device=dev)
    if workspace is None:
        workspace = torch.empty(fastgl_idmap_workspace_bytes(n_dst, n_nbr), dtype=torch.uint8, device=dev)
    _dev(local_nbr, torch.int32, "local_nbr")
    _dev(unique_gid, torch.int64, "unique_gid")
    _dev(result, torch.int32, "result")
    if local_nbr.numel() < n_nbr or unique_gid.numel() < n_dst + n_nbr or result.numel() < 2:
        raise ValueError("output arrays too small")
    _check(lib().fastgl_idmap(_ptr(dst_gid), n_dst, _ptr(nbr_gid), n_nbr, IDMAP_MODES[mode], _ptr(local_nbr),
                              _ptr(unique_gid), _ptr(result), _ptr(workspace), workspace.numel(), _stream()))
    return local_nbr, unique_gid, result


def fastgl_match_workspace_bytes(n_prev: int, n_new: int) -> int:
    return int(lib().fastgl_match_workspace_bytes(n_prev, n_new))


def fastgl_match(prev_gid: torch.Tensor, new_gid: torch.Tensor, src_row=None, load_pos=None, load_gid=None,
                 result=None, workspace=None):
    """Returns (src_row int32[n_new], load_pos int32[n_new], load_gid int64[n_new], result int32[2]) on
    the device, nothing synchronised: result[0] = rows to load, result[1] = violations."""
    _dev(prev_gid, torch.int64, "prev_gid")
    _dev(new_gid, torch.int64, "new_gid")
    n_prev, n_new, dev = prev_gid.numel(), new_gid.numel(), new_gid.device
    src_row = torch.empty(n_new, dtype=torch.int32, device=dev) if src_row is None else src_row
    load_pos = torch.empty(n_new, dtype=torch.int32, device=dev) if load_pos is None else load_pos
    load_gid = torch.empty(n_new, dtype=torch.int64, device=dev) if load_gid is None else load_gid
    result = torch.empty(2, dtype=torch.int32, device=dev) if result is None else result
    if workspace is None:
        workspace = torch.empty(fastgl_match_workspace_bytes(n_prev, n_new), dtype=torch.uint8, device=dev)
    _dev(src_row, torch.int32, "src_row")
    _dev(load_pos, torch.int32, "load_pos")
    _dev(load_gid, torch.int64, "load_gid")
    _dev(result, torch.int32, "result")
    if min(src_row.numel(), load_pos.numel(), load_gid.numel()) < n_new or result.numel() < 2:
        raise ValueError("output arrays too small")
    _check(lib().fastgl_match(_ptr(prev_gid), n_prev, _ptr(new_gid), n_new, _ptr(src_row), _ptr(load_pos),
                              _ptr(load_gid), _ptr(result), _ptr(workspace), workspace.numel(), _stream()))
    return src_row, load_pos, load_gid, result


def fastgl_assemble_rows(X_prev: torch.Tensor, X_load: torch.Tensor, src_row: torch.Tensor, n_load: int,
                         out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """X_load may have more rows than n_load (a buffer sized for the worst case); the first n_load count."""
    dt = _feat_dtype(X_prev)
    _dev(X_prev, X_prev.dtype, "X_prev")
    _dev(X_load, X_prev.dtype, "X_load")
    _dev(src_row, torch.int32, "src_row")
    feat, n_new = X_prev.shape[1], src_row.numel()
    if X_load.shape[1] != feat or X_load.shape[0] < n_load:
        raise ValueError("X_load must be [>= n_load, feat]")
    if out is None:
        out = torch.empty((n_new, feat), dtype=X_prev.dtype, device=X_prev.device)
    _dev(out, X_prev.dtype, "out")
    if tuple(out.shape) != (n_new, feat):
        raise ValueError("out must be [n_new, feat]")
    _check(lib().fastgl_assemble_rows(_ptr(X_prev), X_prev.shape[0], _ptr(X_load), n_load, _ptr(src_row), n_new,
                                      feat, dt, _ptr(out), _stream()))
    return out


def fastgl_overlap_workspace_bytes(total_ids: int) -> int:
    return int(lib().fastgl_overlap_workspace_bytes(total_ids))


def fastgl_overlap_counts(gid: torch.Tensor, offsets, workspace: Optional[torch.Tensor] = None):
    """gid: the node lists of n mini-batches one after the other (device int64); offsets: n+1 host
    ints.  Returns (counts int64[n,n], violations int32[1]) on the device."""
    _dev(gid, torch.int64, "gid")
    n = len(offsets) - 1
    off = (ctypes.c_int64 * (n + 1))(*[int(x) for x in offsets])
    counts = torch.empty((n, n), dtype=torch.int64, device=gid.device)
    viol = torch.empty(1, dtype=torch.int32, device=gid.device)
    if workspace is None:
        workspace = torch.empty(fastgl_overlap_workspace_bytes(gid.numel()), dtype=torch.uint8, device=gid.device)
    _check(lib().fastgl_overlap_counts(_ptr(gid), off, n, _ptr(counts), _ptr(viol), _ptr(workspace),
                                       workspace.numel(), _stream()))
    return counts, viol


def fastgl_greedy_reorder(overlap, sizes):
    """Host-side Algorithm 1: overlap = n x n nested sequence / array of ints, sizes = n ints."""
    n = len(sizes)
    flat = [int(x) for row in overlap for x in row]
    if len(flat) != n * n:
        raise ValueError("overlap must be n x n")
    ov = (ctypes.c_int64 * max(n * n, 1))(*flat)
    sz_ = (ctypes.c_int64 * max(n, 1))(*[int(x) for x in sizes])
    order = (ctypes.c_int32 * max(n, 1))()
    _check(lib().fastgl_greedy_reorder(ov, sz_, n, order))
    return [int(order[i]) for i in range(n)]


def fastgl_edge_workspace_bytes(num_dst: int, num_edges: int) -> int:
    return int(lib().fastgl_edge_workspace_bytes(num_dst, num_edges))


def fastgl_edge_softmax_long_row() -> int:
    return int(lib().fastgl_edge_softmax_long_row())


def _edge_ws(indptr, num_edges, workspace):
    if workspace is None:
        workspace = torch.empty(fastgl_edge_workspace_bytes(indptr.numel() - 1, num_edges), dtype=torch.uint8,
                                device=indptr.device)
    return workspace


def fastgl_edge_weight_grad(indptr, indices, num_src: int, mode: str, X: torch.Tensor, grad_out: torch.Tensor,
                            plan: Optional[Plan] = None, grad_w: Optional[torch.Tensor] = None,
                            workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    _dev(indptr, torch.int32, "indptr")
    _dev(indices, torch.int32, "indices")
    dt = _feat_dtype(X)
    _dev(X, X.dtype, "X")
    _dev(grad_out, X.dtype, "grad_out")
    num_dst, num_edges, feat = indptr.numel() - 1, indices.numel(), X.shape[1]
    if X.shape[0] != num_src or tuple(grad_out.shape) != (num_dst, feat):
        raise ValueError("X must be [num_src, feat] and grad_out [num_dst, feat]")
    if grad_w is None:
        grad_w = torch.empty(num_edges, dtype=torch.float32, device=X.device)
    _dev(grad_w, torch.float32, "grad_w")
    if grad_w.numel() != num_edges:
        raise ValueError("grad_w must have one entry per edge")
    workspace = _edge_ws(indptr, num_edges, workspace)
    _check(lib().fastgl_edge_weight_grad(_ptr(indptr), _ptr(indices), num_dst, num_src, num_edges, feat, MODES[mode],
                                         dt, _ptr(X), _ptr(grad_out), plan.handle if plan is not None else None,
                                         _ptr(grad_w), _ptr(workspace), workspace.numel(), _stream()))
    return grad_w


def fastgl_edge_softmax_fwd(indptr, score: torch.Tensor, alpha: Optional[torch.Tensor] = None,
                            workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    _dev(indptr, torch.int32, "indptr")
    _dev(score, torch.float32, "score")
    alpha = torch.empty_like(score) if alpha is None else alpha
    _dev(alpha, torch.float32, "alpha")
    if alpha.numel() != score.numel():
        raise ValueError("alpha must have one entry per edge")
    workspace = _edge_ws(indptr, score.numel(), workspace)
    _check(lib().fastgl_edge_softmax_fwd(_ptr(indptr), indptr.numel() - 1, score.numel(), _ptr(score), _ptr(alpha),
                                         _ptr(workspace), workspace.numel(), _stream()))
    return alpha


def fastgl_edge_softmax_bwd(indptr, alpha: torch.Tensor, grad_alpha: torch.Tensor,
                            grad_score: Optional[torch.Tensor] = None,
                            workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    _dev(indptr, torch.int32, "indptr")
    _dev(alpha, torch.float32, "alpha")
    _dev(grad_alpha, torch.float32, "grad_alpha")
    grad_score = torch.empty_like(alpha) if grad_score is None else grad_score
    _dev(grad_score, torch.float32, "grad_score")
    if grad_alpha.numel() != alpha.numel() or grad_score.numel() != alpha.numel():
        raise ValueError("per-edge arrays must have one entry per edge")
    workspace = _edge_ws(indptr, alpha.numel(), workspace)
    _check(lib().fastgl_edge_softmax_bwd(_ptr(indptr), indptr.numel() - 1, alpha.numel(), _ptr(alpha),
                                         _ptr(grad_alpha), _ptr(grad_score), _ptr(workspace), workspace.numel(),
                                         _stream()))
    return grad_score


def fastgl_edge_score_fwd(indptr, indices, el: torch.Tensor, er: torch.Tensor, slope: float,
                          score: Optional[torch.Tensor] = None) -> torch.Tensor:
    _dev(indptr, torch.int32, "indptr")
    _dev(indices, torch.int32, "indices")
    _dev(el, torch.float32, "el")
    _dev(er, torch.float32, "er")
    num_dst, num_edges = indptr.numel() - 1, indices.numel()
    if el.numel() != num_dst:
        raise ValueError("el must have one entry per destination node")
    if score is None:
        score = torch.empty(num_edges, dtype=torch.float32, device=el.device)
    _dev(score, torch.float32, "score")
    if score.numel() != num_edges:
        raise ValueError("score must have one entry per edge")
    _check(lib().fastgl_edge_score_fwd(_ptr(indptr), _ptr(indices), num_dst, er.numel(), num_edges, _ptr(el), _ptr(er),
                                       float(slope), _ptr(score), _stream()))
    return score


def fastgl_edge_score_bwd(indptr, indices, el: torch.Tensor, er: torch.Tensor, slope: float, grad_score: torch.Tensor,
                          plan: Optional[Plan] = None, want=("el", "er"), grad_el: Optional[torch.Tensor] = None,
                          grad_er: Optional[torch.Tensor] = None):
    """(grad_el, grad_er); `want` selects which are computed when no array is passed in (the other is
    None).  grad_er needs a plan built with PLAN_BWD | PLAN_PERM."""
    _dev(indptr, torch.int32, "indptr")
    _dev(indices, torch.int32, "indices")
    _dev(el, torch.float32, "el")
    _dev(er, torch.float32, "er")
    _dev(grad_score, torch.float32, "grad_score")
    num_dst, num_edges = indptr.numel() - 1, indices.numel()
    if el.numel() != num_dst or grad_score.numel() != num_edges:
        raise ValueError("el must have one entry per destination node, grad_score one per edge")
    g_el = grad_el if grad_el is not None else (torch.empty_like(el) if "el" in want else None)
    g_er = grad_er if grad_er is not None else (torch.empty_like(er) if "er" in want else None)
    for name, g, ref in (("grad_el", g_el, el), ("grad_er", g_er, er)):
        if g is not None:
            _dev(g, torch.float32, name)
            if g.numel() != ref.numel():
                raise ValueError(f"{name} must have one entry per node")
    _check(lib().fastgl_edge_score_bwd(_ptr(indptr), _ptr(indices), num_dst, er.numel(), num_edges, _ptr(el), _ptr(er),
                                       float(slope), _ptr(grad_score), plan.handle if plan is not None else None,
                                       _ptr(g_el), _ptr(g_er), _stream()))
    return g_el, g_er

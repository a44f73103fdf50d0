"""Thin Python binding of libflexshard_hip.so (argument marshalling only).

Every function has the name and the arguments of the C entry point declared in
include/flexshard.h; tensors are torch CUDA tensors whose device pointers are
passed through, the stream is torch's current stream.  Nothing is computed
here, and there is no fallback: without the built library every call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Tuple

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("FLEXSHARD_HIP_LIB", os.path.join(_PKG, "libflexshard_hip.so"))

FS_F32, FS_F16, FS_BF16 = 0, 1, 2
FS_DEV_BAD_ID, FS_DEV_BAD_OFFSETS, FS_DEV_BAD_PLACEMENT = 1, 2, 4
FS_DEV_COUNT_OVERFLOW, FS_DEV_UNIQUE_OVERFLOW, FS_DEV_POS_ORDER, FS_DEV_NOT_SORTED = 8, 16, 32, 64
FS_PLAN_ACCUMULATE, FS_PLAN_SELECT, FS_PLAN_TAG, FS_PLAN_ALLOW_ZERO = 1, 2, 4, 8
FS_BWD_TILE = 256
FS_OPT_SGD, FS_OPT_ADAGRAD_ROWWISE, FS_OPT_ADAGRAD = 0, 1, 2
(FS_CUT_CANDIDATES, FS_CUT_A, FS_CUT_B, FS_CUT_C, FS_CUT_FLEX, FS_CUT_N_DP, FS_CUT_N_FLEX, FS_CUT_SUM_ALL,
 FS_CUT_SUM_DP, FS_CUT_SUM_FLEX) = range(10)
FS_TIER_CUTS = 10
FS_MAX_BUCKETS = 4096
FS_ROUTE_NOALLOC_SCRATCH_BYTES = 32 << 20

STATUS_NAMES = {0: "FS_OK", 1: "FS_ERR_NULL", 2: "FS_ERR_SIZE", 3: "FS_ERR_DTYPE", 4: "FS_ERR_ALIGN",
                5: "FS_ERR_WORKSPACE", 6: "FS_ERR_CONFIG", 7: "FS_ERR_DEVICE"}

EXPORTS = ["fs_route_bucketize", "fs_route_bucketize_noalloc", "fs_seq_gather_fwd", "fs_seq_grad_bwd", "fs_plan_replication",
           "fs_sort_lookups", "fs_seq_grad_bwd_sorted", "fs_seq_gather_fwd_sorted", "fs_seq_grad_bwd_update",
           "fs_seq_gather_send", "fs_seq_unbucketize", "fs_replica_build", "fs_seq_gather_fwd_replica", "fs_plan_tiers",
           "fs_replica_tag_slots", "fs_route_bucketize_slots", "fs_seq_gather_fwd_slots",
           "fs_cost_model", "fs_tier_traffic", "fs_sparse_update", "fs_util_copy", "fs_util_read_write_mix", "fs_version", "fs_bwd_tile", "fs_prof_begin", "fs_prof_only", "fs_prof_end"]

_DTYPES = {torch.float32: FS_F32, torch.float16: FS_F16, torch.bfloat16: FS_BF16}

_lib: Optional[ctypes.CDLL] = None


class FlexShardError(RuntimeError):
    def __init__(self, fn: str, code: int):
        super().__init__(f"{fn} returned {STATUS_NAMES.get(code, code)}")
        self.code = code


def lib() -> ctypes.CDLL:
    """The loaded HIP library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2301_02959_amd.build` "
                "(hipcc, gfx950); this package has no other code path")
        _lib = ctypes.CDLL(LIB_PATH)
        for name in ("fs_sort_lookups", "fs_seq_grad_bwd_sorted", "fs_seq_gather_fwd_sorted", "fs_seq_grad_bwd_update",
                     "fs_route_bucketize", "fs_route_bucketize_noalloc", "fs_seq_gather_fwd", "fs_seq_grad_bwd", "fs_plan_replication",
                     "fs_seq_gather_send", "fs_seq_unbucketize", "fs_replica_build",
                     "fs_replica_tag_slots", "fs_route_bucketize_slots", "fs_seq_gather_fwd_slots",
                     "fs_seq_gather_fwd_replica", "fs_plan_tiers", "fs_cost_model", "fs_tier_traffic", "fs_sparse_update", "fs_prof_begin", "fs_prof_only",
                     "fs_util_copy", "fs_util_read_write_mix"):
            getattr(_lib, name).restype = ctypes.c_int
        _lib.fs_version.restype = ctypes.c_int32
        _lib.fs_bwd_tile.restype = ctypes.c_int32
        _lib.fs_prof_end.restype = ctypes.c_int32
    return _lib


_I64 = (torch.int64,)
_I32 = (torch.int32,)
_U32 = (torch.int32, torch.uint32)          # 32-bit words: torch code usually holds them as int32
_F32 = (torch.float32,)
_ROWS = (torch.float32, torch.float16, torch.bfloat16)


def _ptr(t: Optional[torch.Tensor], dtypes: Optional[tuple] = None) -> ctypes.c_void_p:
    """Device pointer of a contiguous CUDA tensor (None -> NULL); `dtypes`: the element types the C side reads."""
    if t is None:
        return ctypes.c_void_p(0)
    if not t.is_cuda:
        raise TypeError("the library takes device memory: got a tensor on " + str(t.device))
    if not t.is_contiguous():
        raise TypeError("tensors must be contiguous")
    if dtypes is not None and t.dtype not in dtypes:
        raise TypeError(f"expected a tensor of {' or '.join(str(d) for d in dtypes)}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(fn: str, code: int, raise_on_error: bool) -> int:
    if code != 0 and raise_on_error:
        raise FlexShardError(fn, code)
    return code


def _workspace(query, device) -> Tuple[Optional[torch.Tensor], ctypes.c_size_t, int]:
    """Ask the entry point for its scratch size, then allocate it through torch."""
    size = ctypes.c_size_t(0)
    code = query(ctypes.c_void_p(0), ctypes.byref(size))
    if code != 0:
        return None, size, code
    ws = torch.empty(max(int(size.value), 256), dtype=torch.uint8, device=device)
    return ws, ctypes.c_size_t(ws.numel()), 0


def fs_route_bucketize(ids, offsets, T: int, B: int, row_base, placement, n: int, U: int, W: int, self_: int,
                       bucket_offsets, out_rows, out_pos, tier_counts=None, dev_status=None,
                       workspace: Optional[torch.Tensor] = None, raise_on_error: bool = True) -> int:
    L = lib()

    def call(ws_ptr, ws_size_ref):
        return L.fs_route_bucketize(
            _ptr(ids, _I64), _ptr(offsets, _I64), ctypes.c_int32(T), ctypes.c_int32(B), _ptr(row_base, _I64), _ptr(placement, _U32),
            ctypes.c_int64(n), ctypes.c_int32(U), ctypes.c_int32(W), ctypes.c_int32(self_),
            _ptr(bucket_offsets, _I64), _ptr(out_rows, _I64), _ptr(out_pos, _I32), _ptr(tier_counts, _I64),
            ws_ptr, ws_size_ref, _stream(), _ptr(dev_status, _I32))

    if workspace is None:
        workspace, size, code = _workspace(call, offsets.device)
        if code != 0:
            return _check("fs_route_bucketize", code, raise_on_error)
    else:
        size = ctypes.c_size_t(workspace.numel())
    return _check("fs_route_bucketize", call(_ptr(workspace), ctypes.byref(size)), raise_on_error)


def fs_route_bucketize_noalloc(ids, offsets, T: int, B: int, row_base, placement, n: int, U: int, W: int, self_: int,
                               bucket_offsets, out_rows, out_pos, tier_counts=None, dev_status=None,
                               raise_on_error: bool = True) -> int:
    code = lib().fs_route_bucketize_noalloc(
        _ptr(ids, _I64), _ptr(offsets, _I64), ctypes.c_int32(T), ctypes.c_int32(B), _ptr(row_base, _I64), _ptr(placement, _U32),
        ctypes.c_int64(n), ctypes.c_int32(U), ctypes.c_int32(W), ctypes.c_int32(self_),
        _ptr(bucket_offsets, _I64), _ptr(out_rows, _I64), _ptr(out_pos, _I32), _ptr(tier_counts, _I64),
        _stream(), _ptr(dev_status, _I32))
    return _check("fs_route_bucketize_noalloc", code, raise_on_error)


def route_workspace_bytes(T: int, B: int, n: int, U: int, W: int, self_: int) -> int:
    size = ctypes.c_size_t(0)
    z = ctypes.c_void_p(0)
    code = lib().fs_route_bucketize(z, z, ctypes.c_int32(T), ctypes.c_int32(B), z, z, ctypes.c_int64(n),
                                    ctypes.c_int32(U), ctypes.c_int32(W), ctypes.c_int32(self_), z, z, z, z,
                                    z, ctypes.byref(size), z, z)
    _check("fs_route_bucketize", code, True)
    return int(size.value)


def fs_seq_gather_fwd(weights, rows, pos, j0: int, j1: int, out, dev_status=None,
                      raise_on_error: bool = True, R: Optional[int] = None, D: Optional[int] = None,
                      dtype: Optional[int] = None, n: Optional[int] = None) -> int:
    R = weights.shape[0] if R is None else R
    D = weights.shape[1] if D is None else D
    n = out.shape[0] if n is None else n
    dtype = _DTYPES[weights.dtype] if dtype is None else dtype
    code = lib().fs_seq_gather_fwd(
        _ptr(weights, _ROWS), ctypes.c_int64(R), ctypes.c_int32(D), ctypes.c_int(dtype), _ptr(rows, _I64), _ptr(pos, _I32),
        ctypes.c_int64(j0), ctypes.c_int64(j1), _ptr(out, _ROWS), ctypes.c_int64(n), _stream(), _ptr(dev_status, _I32))
    return _check("fs_seq_gather_fwd", code, raise_on_error)


def fs_seq_gather_send(weights, rows, j0: int, j1: int, send, dev_status=None, raise_on_error: bool = True,
                       R: Optional[int] = None, D: Optional[int] = None, dtype: Optional[int] = None) -> int:
    R = weights.shape[0] if R is None else R
    D = weights.shape[1] if D is None else D
    dtype = _DTYPES[weights.dtype] if dtype is None else dtype
    code = lib().fs_seq_gather_send(
        _ptr(weights, _ROWS), ctypes.c_int64(R), ctypes.c_int32(D), ctypes.c_int(dtype), _ptr(rows, _I64),
        ctypes.c_int64(j0), ctypes.c_int64(j1), _ptr(send, _ROWS), _stream(), _ptr(dev_status, _I32))
    return _check("fs_seq_gather_send", code, raise_on_error)


def fs_seq_unbucketize(recv, pos, j0: int, j1: int, out, dev_status=None, raise_on_error: bool = True,
                       D: Optional[int] = None, dtype: Optional[int] = None, n: Optional[int] = None) -> int:
    D = recv.shape[1] if D is None else D
    n = out.shape[0] if n is None else n
    dtype = _DTYPES[recv.dtype] if dtype is None else dtype
    code = lib().fs_seq_unbucketize(
        _ptr(recv, _ROWS), ctypes.c_int32(D), ctypes.c_int(dtype), _ptr(pos, _I32), ctypes.c_int64(j0), ctypes.c_int64(j1),
        _ptr(out, _ROWS), ctypes.c_int64(n), _stream(), _ptr(dev_status, _I32))
    return _check("fs_seq_unbucketize", code, raise_on_error)


def fs_replica_build(weights, sel_rows, k: int, num_selected, store, slot_of_row, dev_status=None,
                     raise_on_error: bool = True, R: Optional[int] = None, D: Optional[int] = None,
                     dtype: Optional[int] = None) -> int:
    R = weights.shape[0] if R is None else R
    D = weights.shape[1] if D is None else D
    dtype = _DTYPES[weights.dtype] if dtype is None else dtype
    code = lib().fs_replica_build(
        _ptr(weights, _ROWS), ctypes.c_int64(R), ctypes.c_int32(D), ctypes.c_int(dtype), _ptr(sel_rows, _I64),
        ctypes.c_int64(k), _ptr(num_selected, _I64), _ptr(store, _ROWS), _ptr(slot_of_row, _I32), _stream(), _ptr(dev_status, _I32))
    return _check("fs_replica_build", code, raise_on_error)


def fs_seq_gather_fwd_replica(weights, store, k: int, slot_of_row, rows, pos, j0: int, j1: int, out,
                              dev_status=None, raise_on_error: bool = True, R: Optional[int] = None,
                              D: Optional[int] = None, dtype: Optional[int] = None,
                              n: Optional[int] = None) -> int:
    R = weights.shape[0] if R is None else R
    D = weights.shape[1] if D is None else D
    n = out.shape[0] if n is None else n
    dtype = _DTYPES[weights.dtype] if dtype is None else dtype
    code = lib().fs_seq_gather_fwd_replica(
        _ptr(weights, _ROWS), ctypes.c_int64(R), ctypes.c_int32(D), ctypes.c_int(dtype), _ptr(store, _ROWS), ctypes.c_int64(k),
        _ptr(slot_of_row, _I32), _ptr(rows, _I64), _ptr(pos, _I32), ctypes.c_int64(j0), ctypes.c_int64(j1), _ptr(out, _ROWS),
        ctypes.c_int64(n), _stream(), _ptr(dev_status, _I32))
    return _check("fs_seq_gather_fwd_replica", code, raise_on_error)


def fs_replica_tag_slots(placement, slot_of_row, dev_status=None, raise_on_error: bool = True,
                         R: Optional[int] = None) -> int:
    R = placement.shape[0] if R is None else R
    code = lib().fs_replica_tag_slots(_ptr(placement, _U32), ctypes.c_int64(R), _ptr(slot_of_row, _I32), _stream(),
                                      _ptr(dev_status, _I32))
    return _check("fs_replica_tag_slots", code, raise_on_error)


def fs_route_bucketize_slots(ids, offsets, T: int, B: int, row_base, placement, n: int, U: int, W: int, self_: int,
                             bucket_offsets, out_rows, out_pos, out_slots, tier_counts=None, dev_status=None,
                             workspace: Optional[torch.Tensor] = None, raise_on_error: bool = True) -> int:
    L = lib()

    def call(ws_ptr, ws_size_ref):
        return L.fs_route_bucketize_slots(
            _ptr(ids, _I64), _ptr(offsets, _I64), ctypes.c_int32(T), ctypes.c_int32(B), _ptr(row_base, _I64), _ptr(placement, _U32),
            ctypes.c_int64(n), ctypes.c_int32(U), ctypes.c_int32(W), ctypes.c_int32(self_),
            _ptr(bucket_offsets, _I64), _ptr(out_rows, _I64), _ptr(out_pos, _I32), _ptr(out_slots, _I32), _ptr(tier_counts, _I64),
            ws_ptr, ws_size_ref, _stream(), _ptr(dev_status, _I32))

    if workspace is None:
        workspace, size, code = _workspace(call, offsets.device)
        if code != 0:
            return _check("fs_route_bucketize_slots", code, raise_on_error)
    else:
        size = ctypes.c_size_t(workspace.numel())
    return _check("fs_route_bucketize_slots", call(_ptr(workspace), ctypes.byref(size)), raise_on_error)


def fs_seq_gather_fwd_slots(weights, store, k: int, rows, slots, pos, j0: int, j1: int, out,
                            dev_status=None, raise_on_error: bool = True, R: Optional[int] = None,
                            D: Optional[int] = None, dtype: Optional[int] = None, n: Optional[int] = None) -> int:
    R = weights.shape[0] if R is None else R
    D = weights.shape[1] if D is None else D
    n = out.shape[0] if n is None else n
    dtype = _DTYPES[weights.dtype] if dtype is None else dtype
    code = lib().fs_seq_gather_fwd_slots(
        _ptr(weights, _ROWS), ctypes.c_int64(R), ctypes.c_int32(D), ctypes.c_int(dtype), _ptr(store, _ROWS), ctypes.c_int64(k),
        _ptr(rows, _I64), _ptr(slots, _I32), _ptr(pos, _I32), ctypes.c_int64(j0), ctypes.c_int64(j1), _ptr(out, _ROWS),
        ctypes.c_int64(n), _stream(), _ptr(dev_status, _I32))
    return _check("fs_seq_gather_fwd_slots", code, raise_on_error)


def fs_seq_grad_bwd(grad_out, rows, pos, j0: int, j1: int, R: int, variant: int,
                    uniq_rows, row_grads, cap_unique: int, num_unique, dev_status=None,
                    workspace: Optional[torch.Tensor] = None, raise_on_error: bool = True,
                    n: Optional[int] = None, D: Optional[int] = None, dtype: Optional[int] = None) -> int:
    L = lib()
    n = grad_out.shape[0] if n is None else n
    D = grad_out.shape[1] if D is None else D
    dtype = _DTYPES[grad_out.dtype] if dtype is None else dtype

    def call(ws_ptr, ws_size_ref):
        return L.fs_seq_grad_bwd(
            _ptr(grad_out, _ROWS), ctypes.c_int64(n), ctypes.c_int32(D), ctypes.c_int(dtype), _ptr(rows, _I64), _ptr(pos, _I32),
            ctypes.c_int64(j0), ctypes.c_int64(j1), ctypes.c_int64(R), ctypes.c_int32(variant),
            _ptr(uniq_rows, _I64), _ptr(row_grads, _F32), ctypes.c_int64(cap_unique), _ptr(num_unique, _I64),
            ws_ptr, ws_size_ref, _stream(), _ptr(dev_status, _I32))

    if workspace is None:
        workspace, size, code = _workspace(call, grad_out.device)
        if code != 0:
            return _check("fs_seq_grad_bwd", code, raise_on_error)
    else:
        size = ctypes.c_size_t(workspace.numel())
    return _check("fs_seq_grad_bwd", call(_ptr(workspace), ctypes.byref(size)), raise_on_error)


def fs_sort_lookups(rows, pos, j0: int, j1: int, R: int, n: int, sorted_rows, sorted_pos, dev_status=None,
                    workspace: Optional[torch.Tensor] = None, raise_on_error: bool = True) -> int:
    L = lib()

    def call(ws_ptr, ws_size_ref):
        return L.fs_sort_lookups(_ptr(rows, _I64), _ptr(pos, _I32), ctypes.c_int64(j0), ctypes.c_int64(j1), ctypes.c_int64(R),
                                 ctypes.c_int64(n), _ptr(sorted_rows, _U32), _ptr(sorted_pos, _U32), ws_ptr, ws_size_ref,
                                 _stream(), _ptr(dev_status, _I32))

    if workspace is None:
        device = next((t.device for t in (rows, sorted_rows, pos) if t is not None), "cuda")
        workspace, size, code = _workspace(call, device)
        if code != 0:
            return _check("fs_sort_lookups", code, raise_on_error)
    else:
        size = ctypes.c_size_t(workspace.numel())
    return _check("fs_sort_lookups", call(_ptr(workspace), ctypes.byref(size)), raise_on_error)


def fs_seq_grad_bwd_sorted(grad_out, sorted_rows, sorted_pos, m: int, R: int, variant: int,
                           uniq_rows, row_grads, cap_unique: int, num_unique, dev_status=None,
                           workspace: Optional[torch.Tensor] = None, raise_on_error: bool = True,
                           n: Optional[int] = None, D: Optional[int] = None, dtype: Optional[int] = None) -> int:
    L = lib()
    n = grad_out.shape[0] if n is None else n
    D = grad_out.shape[1] if D is None else D
    dtype = _DTYPES[grad_out.dtype] if dtype is None else dtype

    def call(ws_ptr, ws_size_ref):
        return L.fs_seq_grad_bwd_sorted(
            _ptr(grad_out, _ROWS), ctypes.c_int64(n), ctypes.c_int32(D), ctypes.c_int(dtype), _ptr(sorted_rows, _U32),
            _ptr(sorted_pos, _U32), ctypes.c_int64(m), ctypes.c_int64(R), ctypes.c_int32(variant),
            _ptr(uniq_rows, _I64), _ptr(row_grads, _F32), ctypes.c_int64(cap_unique), _ptr(num_unique, _I64),
            ws_ptr, ws_size_ref, _stream(), _ptr(dev_status, _I32))

    if workspace is None:
        workspace, size, code = _workspace(call, grad_out.device)
        if code != 0:
            return _check("fs_seq_grad_bwd_sorted", code, raise_on_error)
    else:
        size = ctypes.c_size_t(workspace.numel())
    return _check("fs_seq_grad_bwd_sorted", call(_ptr(workspace), ctypes.byref(size)), raise_on_error)


def fs_seq_gather_fwd_sorted(weights, sorted_rows, sorted_pos, m: int, out, dev_status=None,
                             raise_on_error: bool = True, R: Optional[int] = None, D: Optional[int] = None,
                             dtype: Optional[int] = None, n: Optional[int] = None) -> int:
    R = weights.shape[0] if R is None else R
    D = weights.shape[1] if D is None else D
    n = out.shape[0] if n is None else n
    dtype = _DTYPES[weights.dtype] if dtype is None else dtype
    code = lib().fs_seq_gather_fwd_sorted(
        _ptr(weights, _ROWS), ctypes.c_int64(R), ctypes.c_int32(D), ctypes.c_int(dtype), _ptr(sorted_rows, _U32),
        _ptr(sorted_pos, _U32), ctypes.c_int64(m), _ptr(out, _ROWS), ctypes.c_int64(n), _stream(), _ptr(dev_status, _I32))
    return _check("fs_seq_gather_fwd_sorted", code, raise_on_error)


def fs_plan_replication(ids, offsets, T: int, B: int, row_base, n: int, R: int, counts, flags: int,
                        budget_bytes: int = 0, bytes_per_row: int = 1, sel_rows=None, num_selected=None,
                        placement=None, dev_status=None, workspace: Optional[torch.Tensor] = None,
                        raise_on_error: bool = True) -> int:
    L = lib()

    def call(ws_ptr, ws_size_ref):
        return L.fs_plan_replication(
            _ptr(ids, _I64), _ptr(offsets, _I64), ctypes.c_int32(T), ctypes.c_int32(B), _ptr(row_base, _I64), ctypes.c_int64(n),
            ctypes.c_int64(R), _ptr(counts, _U32), ctypes.c_int32(flags), ctypes.c_int64(budget_bytes),
            ctypes.c_int64(bytes_per_row), _ptr(sel_rows, _I64), _ptr(num_selected, _I64), _ptr(placement, _U32),
            ws_ptr, ws_size_ref, _stream(), _ptr(dev_status, _I32))

    if workspace is None:
        workspace, size, code = _workspace(call, counts.device)
        if code != 0:
            return _check("fs_plan_replication", code, raise_on_error)
    else:
        size = ctypes.c_size_t(workspace.numel())
    return _check("fs_plan_replication", call(_ptr(workspace), ctypes.byref(size)), raise_on_error)


class TierParams(ctypes.Structure):
    """fs_tier_params of the C header, field for field."""
    _fields_ = [("num_samples", ctypes.c_int64), ("B", ctypes.c_int64), ("U", ctypes.c_int32), ("W", ctypes.c_int32),
                ("dp_multiplier", ctypes.c_int32), ("granule", ctypes.c_int32), ("a2a_global", ctypes.c_int64),
                ("a2a_intra", ctypes.c_int64), ("ar_global", ctypes.c_int64), ("ar_cross", ctypes.c_int64)]


def fs_plan_tiers(counts, R: int, params: dict, tiers: int, sorted_rows, cap: int, cuts, placement=None,
                  dev_status=None, workspace: Optional[torch.Tensor] = None, raise_on_error: bool = True) -> int:
    L = lib()
    tp = TierParams(**params)

    def call(ws_ptr, ws_size_ref):
        return L.fs_plan_tiers(_ptr(counts, _U32), ctypes.c_int64(R), ctypes.byref(tp), ctypes.c_int32(tiers),
                               _ptr(sorted_rows, _I64), ctypes.c_int64(cap), _ptr(cuts, _I64), _ptr(placement, _U32),
                               ws_ptr, ws_size_ref, _stream(), _ptr(dev_status, _I32))

    if workspace is None:
        device = next((t.device for t in (counts, cuts, sorted_rows) if t is not None), "cuda")
        workspace, size, code = _workspace(call, device)
        if code != 0:
            return _check("fs_plan_tiers", code, raise_on_error)
    else:
        size = ctypes.c_size_t(workspace.numel())
    return _check("fs_plan_tiers", call(_ptr(workspace), ctypes.byref(size)), raise_on_error)


def fs_sparse_update(weights, uniq_rows, row_grads, cap_unique: int, num_unique, optimizer: int, lr: float, eps: float,
                     state=None, store=None, slot_of_row=None, k: int = 0, dev_status=None,
                     raise_on_error: bool = True, R: Optional[int] = None, D: Optional[int] = None,
                     dtype: Optional[int] = None) -> int:
    R = weights.shape[0] if R is None else R
    D = weights.shape[1] if D is None else D
    dtype = _DTYPES[weights.dtype] if dtype is None else dtype
    code = lib().fs_sparse_update(
        _ptr(weights, _ROWS), ctypes.c_int64(R), ctypes.c_int32(D), ctypes.c_int(dtype), _ptr(uniq_rows, _I64), _ptr(row_grads, _F32),
        ctypes.c_int64(cap_unique), _ptr(num_unique, _I64), ctypes.c_int32(optimizer), ctypes.c_float(lr), ctypes.c_float(eps),
        _ptr(state, _F32), _ptr(store, _ROWS), _ptr(slot_of_row, _I32), ctypes.c_int64(k), _stream(), _ptr(dev_status, _I32))
    return _check("fs_sparse_update", code, raise_on_error)


def fs_seq_grad_bwd_update(grad_out, sorted_rows, sorted_pos, m: int, R: int, weights, optimizer: int, lr: float,
                           eps: float, state, store, slot_of_row, k: int, uniq_rows, row_grads, cap_unique: int,
                           num_unique, dev_status=None, workspace: Optional[torch.Tensor] = None,
                           raise_on_error: bool = True, n: Optional[int] = None, D: Optional[int] = None,
                           dtype: Optional[int] = None) -> int:
    L = lib()
    n = grad_out.shape[0] if n is None else n
    D = grad_out.shape[1] if D is None else D
    dtype = _DTYPES[grad_out.dtype] if dtype is None else dtype

    def call(ws_ptr, ws_size_ref):
        return L.fs_seq_grad_bwd_update(
            _ptr(grad_out, _ROWS), ctypes.c_int64(n), ctypes.c_int32(D), ctypes.c_int(dtype), _ptr(sorted_rows, _U32),
            _ptr(sorted_pos, _U32), ctypes.c_int64(m), ctypes.c_int64(R), _ptr(weights, _ROWS), ctypes.c_int32(optimizer),
            ctypes.c_float(lr), ctypes.c_float(eps), _ptr(state, _F32), _ptr(store, _ROWS), _ptr(slot_of_row, _I32),
            ctypes.c_int64(k), _ptr(uniq_rows, _I64), _ptr(row_grads, _F32), ctypes.c_int64(cap_unique),
            _ptr(num_unique, _I64), ws_ptr, ws_size_ref, _stream(), _ptr(dev_status, _I32))

    if workspace is None:
        workspace, size, code = _workspace(call, grad_out.device)
        if code != 0:
            return _check("fs_seq_grad_bwd_update", code, raise_on_error)
    else:
        size = ctypes.c_size_t(workspace.numel())
    return _check("fs_seq_grad_bwd_update", call(_ptr(workspace), ctypes.byref(size)), raise_on_error)


class CostParams(ctypes.Structure):
    """fs_cost_params of the C header, field for field."""
    _fields_ = [(k, ctypes.c_double) for k in ("E", "D", "dtype_bytes", "L", "W", "N", "B", "a2a_global", "a2a_intra",
                                               "ar_global", "ar_cross", "dp_multiplier")]


FS_STRATEGY_RW, FS_STRATEGY_CW, FS_STRATEGY_DP, FS_STRATEGY_FLEX = 0, 1, 2, 3


def fs_cost_model(params: dict, strategy: int, raise_on_error: bool = True):
    """Returns (code, [static memory, input dist, rows accessed, dynamic memory, dynamic comm, static comm])."""
    cp = CostParams(**{k: float(v) for k, v in params.items()})
    out = (ctypes.c_double * 6)()
    code = lib().fs_cost_model(ctypes.byref(cp), ctypes.c_int32(strategy), out)
    return _check("fs_cost_model", code, raise_on_error), list(out)


def fs_tier_traffic(tier_counts, D: int, dtype_bytes: int, raise_on_error: bool = True):
    """tier_counts: three host integers.  Returns (code, [all sharded, global left, intra-group, share avoided])."""
    tc = (ctypes.c_int64 * 3)(*[int(x) for x in tier_counts])
    out = (ctypes.c_double * 4)()
    code = lib().fs_tier_traffic(tc, ctypes.c_int32(D), ctypes.c_int32(dtype_bytes), out)
    return _check("fs_tier_traffic", code, raise_on_error), list(out)


def fs_util_copy(dst, src, nbytes: Optional[int] = None, raise_on_error: bool = True) -> int:
    nbytes = src.numel() * src.element_size() if nbytes is None else nbytes
    code = lib().fs_util_copy(_ptr(dst), _ptr(src), ctypes.c_int64(nbytes), _stream())
    return _check("fs_util_copy", code, raise_on_error)


def fs_util_read_write_mix(src, pieces_per_write: int, dst=None, raise_on_error: bool = True) -> int:
    code = lib().fs_util_read_write_mix(_ptr(src), ctypes.c_int64(src.numel() * src.element_size()),
                                        ctypes.c_int32(pieces_per_write), _ptr(dst),
                                        ctypes.c_int64(0 if dst is None else dst.numel() * dst.element_size()), _stream())
    return _check("fs_util_read_write_mix", code, raise_on_error)


def fs_version() -> int:
    return int(lib().fs_version())


def fs_bwd_tile() -> int:
    return int(lib().fs_bwd_tile())


def fs_prof_only(names: Optional[str]) -> None:
    """Restricts the timing to the kernels named (comma-separated); None or "" = every kernel."""
    _check("fs_prof_only", lib().fs_prof_only((names or "").encode()), True)


def fs_prof_begin(max_records: int = 4096, only: Optional[str] = None) -> None:
    """Times every later launch, or only the kernels named in `only` (comma-separated)."""
    fs_prof_only(only)
    _check("fs_prof_begin", lib().fs_prof_begin(ctypes.c_int32(max_records)), True)


def fs_prof_end(cap: int = 4096) -> List[Tuple[str, float]]:
    names = ctypes.create_string_buffer(cap * 48)
    ms = (ctypes.c_float * cap)()
    k = lib().fs_prof_end(names, ms, ctypes.c_int32(cap))
    raw = names.raw
    return [(raw[i * 48:(i + 1) * 48].split(b"\0")[0].decode(), float(ms[i])) for i in range(k)]

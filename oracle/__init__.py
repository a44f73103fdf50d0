"""CPU oracle of the tiered sequence-embedding lookup -- TEST INFRASTRUCTURE.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It wraps oracle/flexshard_oracle.c (plain C, one thread, built
with gcc) through ctypes and takes / returns numpy arrays.  Nothing here is
shared with the HIP library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "flexshard_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

F32, F16, BF16 = 0, 1, 2
BAD_ID, BAD_OFFSETS, BAD_PLACEMENT, COUNT_OVERFLOW, UNIQUE_OVERFLOW, POS_ORDER = 1, 2, 4, 8, 16, 32
NOT_SORTED = 64
PLAN_ACCUMULATE, PLAN_SELECT, PLAN_TAG, PLAN_ALLOW_ZERO = 1, 2, 4, 8
BWD_TILE = 256
OPT_SGD, OPT_ADAGRAD_ROWWISE, OPT_ADAGRAD = 0, 1, 2
CUT_CANDIDATES, CUT_A, CUT_B, CUT_C, CUT_FLEX, CUT_N_DP, CUT_N_FLEX, CUT_SUM_ALL, CUT_SUM_DP, CUT_SUM_FLEX = range(10)
N_CUTS = 10


def build(force: bool = False) -> str:
    """Compile the oracle with gcc; -ffp-contract=off keeps every add unfused."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
               "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _p(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.c_void_p(0)
    assert a.flags["C_CONTIGUOUS"]
    return ctypes.c_void_p(a.ctypes.data)


def _i64(x) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.int64)


def route_bucketize(ids, offsets, T: int, B: int, row_base, placement, U: int, W: int, self_: int,
                    n: Optional[int] = None):
    """Returns (rc, status, bucket_offsets[U+1], out_rows[n], out_pos[n], tier_counts[3])."""
    ids = _i64(ids)
    offsets = _i64(offsets)
    row_base = _i64(row_base)
    placement = np.ascontiguousarray(placement, dtype=np.uint32)
    if n is None:
        n = int(offsets[-1])
    bucket_offsets = np.zeros(max(U, 0) + 1, dtype=np.int64)
    out_rows = np.full(max(n, 0), -1, dtype=np.int64)
    out_pos = np.full(max(n, 0), -1, dtype=np.int32)
    tier_counts = np.zeros(3, dtype=np.int64)
    status = ctypes.c_int32(0)
    rc = lib().oracle_route_bucketize(
        _p(ids), _p(offsets), ctypes.c_int32(T), ctypes.c_int32(B), _p(row_base), _p(placement),
        ctypes.c_int64(n), ctypes.c_int32(U), ctypes.c_int32(W), ctypes.c_int32(self_),
        _p(bucket_offsets), _p(out_rows), _p(out_pos), _p(tier_counts), ctypes.byref(status))
    return rc, status.value, bucket_offsets, out_rows, out_pos, tier_counts


def _dtype_code(a: np.ndarray, dtype: Optional[int]) -> int:
    if dtype is not None:
        return dtype
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.float16:
        return F16
    raise ValueError("pass dtype=BF16 with a uint16 array for bfloat16")


def seq_gather_fwd(weights: np.ndarray, rows, pos, j0: int, j1: int, out: np.ndarray,
                   dtype: Optional[int] = None) -> Tuple[int, int]:
    """out[pos[j], :] = weights[rows[j], :] for j in [j0, j1), in place.  Returns (rc, status)."""
    code = _dtype_code(weights, dtype)
    rows = _i64(rows)
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    R, D = weights.shape
    n = out.shape[0]
    status = ctypes.c_int32(0)
    rc = lib().oracle_seq_gather_fwd(
        _p(weights), ctypes.c_int64(R), ctypes.c_int32(D), ctypes.c_int(code), _p(rows), _p(pos),
        ctypes.c_int64(j0), ctypes.c_int64(j1), _p(out), ctypes.c_int64(n), ctypes.byref(status))
    return rc, status.value


def seq_gather_send(weights: np.ndarray, rows, j0: int, j1: int, send: np.ndarray,
                    dtype: Optional[int] = None) -> Tuple[int, int]:
    """send[j - j0, :] = weights[rows[j], :] for j in [j0, j1), in place.  Returns (rc, status)."""
    code = _dtype_code(weights, dtype)
    rows = _i64(rows)
    R, D = weights.shape
    status = ctypes.c_int32(0)
    rc = lib().oracle_seq_gather_send(
        _p(weights), ctypes.c_int64(R), ctypes.c_int32(D), ctypes.c_int(code), _p(rows),
        ctypes.c_int64(j0), ctypes.c_int64(j1), _p(send), ctypes.byref(status))
    return rc, status.value


def seq_unbucketize(recv: np.ndarray, pos, j0: int, j1: int, out: np.ndarray,
                    dtype: Optional[int] = None) -> Tuple[int, int]:
    """out[pos[j], :] = recv[j - j0, :] for j in [j0, j1), in place.  Returns (rc, status)."""
    code = _dtype_code(recv, dtype)
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    D = recv.shape[1]
    status = ctypes.c_int32(0)
    rc = lib().oracle_seq_unbucketize(
        _p(recv), ctypes.c_int32(D), ctypes.c_int(code), _p(pos), ctypes.c_int64(j0), ctypes.c_int64(j1),
        _p(out), ctypes.c_int64(out.shape[0]), ctypes.byref(status))
    return rc, status.value


def replica_build(weights: np.ndarray, sel_rows, store: np.ndarray, dtype: Optional[int] = None):
    """store[s] = weights[sel_rows[s]] in place.  Returns (rc, status, slot_of_row[R] int32)."""
    code = _dtype_code(weights, dtype)
    sel = _i64(sel_rows)
    R, D = weights.shape
    slots = np.full(R, -7, dtype=np.int32)
    status = ctypes.c_int32(0)
    rc = lib().oracle_replica_build(
        _p(weights), ctypes.c_int64(R), ctypes.c_int32(D), ctypes.c_int(code), _p(sel),
        ctypes.c_int64(sel.shape[0]), _p(store), _p(slots), ctypes.byref(status))
    return rc, status.value, slots


def seq_gather_fwd_replica(weights: np.ndarray, store: np.ndarray, slot_of_row, rows, pos, j0: int, j1: int,
                           out: np.ndarray, dtype: Optional[int] = None) -> Tuple[int, int]:
    """seq_gather_fwd with rows that have a slot read from `store`.  Returns (rc, status)."""
    code = _dtype_code(weights, dtype)
    rows = _i64(rows)
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    slots = np.ascontiguousarray(slot_of_row, dtype=np.int32)
    R, D = weights.shape
    status = ctypes.c_int32(0)
    rc = lib().oracle_seq_gather_fwd_replica(
        _p(weights), ctypes.c_int64(R), ctypes.c_int32(D), ctypes.c_int(code), _p(store),
        ctypes.c_int64(store.shape[0]), _p(slots), _p(rows), _p(pos), ctypes.c_int64(j0), ctypes.c_int64(j1),
        _p(out), ctypes.c_int64(out.shape[0]), ctypes.byref(status))
    return rc, status.value


NO_SLOT = 0x3FFFFFFF


def replica_tag_slots(placement: np.ndarray, slot_of_row) -> Tuple[int, int]:
    """Owner bits of every tier-0 entry of `placement` (uint32, in place) = the row's slot, NO_SLOT if none."""
    assert placement.dtype == np.uint32 and placement.flags.c_contiguous
    slots = np.ascontiguousarray(slot_of_row, dtype=np.int32)
    status = ctypes.c_int32(0)
    rc = lib().oracle_replica_tag_slots(_p(placement), ctypes.c_int64(placement.shape[0]), _p(slots), ctypes.byref(status))
    return rc, status.value


def lookup_slots(placement: np.ndarray, rows, j0: int, j1: int):
    """Returns (rc, status, out_slots[len(rows)] int32): the slot each lookup's placement entry carries over [j0, j1),
    -1 where it has none; entries outside the range keep the sentinel -7."""
    rows = _i64(rows)
    pl = np.ascontiguousarray(placement, dtype=np.uint32)
    out = np.full(rows.shape[0], -7, dtype=np.int32)
    status = ctypes.c_int32(0)
    rc = lib().oracle_lookup_slots(_p(pl), ctypes.c_int64(pl.shape[0]), _p(rows), ctypes.c_int64(j0), ctypes.c_int64(j1),
                                   _p(out), ctypes.byref(status))
    return rc, status.value, out


def seq_gather_fwd_slots(weights: np.ndarray, store: np.ndarray, rows, slots, pos, j0: int, j1: int,
                         out: np.ndarray, dtype: Optional[int] = None) -> Tuple[int, int]:
    """seq_gather_fwd with lookup j read from store[slots[j]] where slots[j] >= 0.  Returns (rc, status)."""
    code = _dtype_code(weights, dtype)
    rows = _i64(rows)
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    slots = np.ascontiguousarray(slots, dtype=np.int32)
    R, D = weights.shape
    status = ctypes.c_int32(0)
    rc = lib().oracle_seq_gather_fwd_slots(
        _p(weights), ctypes.c_int64(R), ctypes.c_int32(D), ctypes.c_int(code), _p(store),
        ctypes.c_int64(store.shape[0]), _p(rows), _p(slots), _p(pos), ctypes.c_int64(j0), ctypes.c_int64(j1),
        _p(out), ctypes.c_int64(out.shape[0]), ctypes.byref(status))
    return rc, status.value


def seq_grad_bwd(grad_out: np.ndarray, rows, pos, j0: int, j1: int, R: int, tile: int = BWD_TILE,
                 cap_unique: Optional[int] = None, dtype: Optional[int] = None, want64: bool = True):
    """Returns (rc, status, uniq_rows[n_u], row_grads[n_u, D] f32, row_grads64 or None, n_u)."""
    code = _dtype_code(grad_out, dtype)
    rows = _i64(rows)
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    n, D = grad_out.shape
    m = max(j1 - j0, 0)
    cap = m if cap_unique is None else cap_unique
    uniq = np.full(max(cap, 0), -1, dtype=np.int64)
    g32 = np.zeros((max(cap, 0), D), dtype=np.float32)
    g64 = np.zeros((max(cap, 0), D), dtype=np.float64) if want64 else None
    nu = ctypes.c_int64(0)
    status = ctypes.c_int32(0)
    rc = lib().oracle_seq_grad_bwd(
        _p(grad_out), ctypes.c_int64(n), ctypes.c_int32(D), ctypes.c_int(code), _p(rows), _p(pos),
        ctypes.c_int64(j0), ctypes.c_int64(j1), ctypes.c_int64(R), ctypes.c_int32(tile),
        _p(uniq), _p(g32), _p(g64), ctypes.c_int64(cap), ctypes.byref(nu), ctypes.byref(status))
    k = min(int(nu.value), max(cap, 0))
    return rc, status.value, uniq[:k], g32[:k], (g64[:k] if want64 else None), int(nu.value)


def sort_lookups(rows, pos, j0: int, j1: int, R: int, n: int):
    """Returns (rc, status, sorted_rows uint32[m], sorted_pos uint32[m]): the lookups in (row, pos) order."""
    rows = _i64(rows)
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    m = max(j1 - j0, 0)
    srows = np.zeros(m, dtype=np.uint32)
    spos = np.zeros(m, dtype=np.uint32)
    status = ctypes.c_int32(0)
    rc = lib().oracle_sort_lookups(_p(rows), _p(pos), ctypes.c_int64(j0), ctypes.c_int64(j1), ctypes.c_int64(R),
                                   ctypes.c_int64(n), _p(srows), _p(spos), ctypes.byref(status))
    return rc, status.value, srows, spos


def plan_replication(ids, offsets, T: int, B: int, row_base, R: int, counts: np.ndarray, flags: int,
                     budget_bytes: int = 0, bytes_per_row: int = 1,
                     placement: Optional[np.ndarray] = None, n: Optional[int] = None):
    """counts (uint32[R]) and placement are updated in place.  Returns (rc, status, sel_rows[k])."""
    assert counts.dtype == np.uint32
    ids_a = _i64(ids) if ids is not None else None
    off_a = _i64(offsets) if offsets is not None else None
    rb_a = _i64(row_base) if row_base is not None else None
    if n is None:
        n = int(off_a[-1]) if off_a is not None else 0
    cap = 0
    if flags & PLAN_SELECT and bytes_per_row >= 1 and budget_bytes >= 0:
        cap = min(R, budget_bytes // bytes_per_row)
    sel = np.full(cap + 16, -1, dtype=np.int64)      # slack: a selection that is too long must show, not be cut
    nsel = ctypes.c_int64(0)
    status = ctypes.c_int32(0)
    rc = lib().oracle_plan_replication(
        _p(ids_a), _p(off_a), ctypes.c_int32(T), ctypes.c_int32(B), _p(rb_a), ctypes.c_int64(n),
        ctypes.c_int64(R), _p(counts), ctypes.c_int32(flags), ctypes.c_int64(budget_bytes),
        ctypes.c_int64(bytes_per_row), _p(sel), ctypes.byref(nsel), _p(placement), ctypes.byref(status))
    return rc, status.value, sel[:int(nsel.value)]


class TierParams(ctypes.Structure):
    _fields_ = [("num_samples", ctypes.c_int64), ("B", ctypes.c_int64), ("U", ctypes.c_int32), ("W", ctypes.c_int32),
                ("dp_multiplier", ctypes.c_int32), ("granule", ctypes.c_int32), ("a2a_global", ctypes.c_int64),
                ("a2a_intra", ctypes.c_int64), ("ar_global", ctypes.c_int64), ("ar_cross", ctypes.c_int64)]


def plan_tiers(counts: np.ndarray, params: dict, tiers: int, cap: Optional[int] = None,
               placement: Optional[np.ndarray] = None):
    """Returns (rc, cuts[N_CUTS] int64, sorted_rows[n_dp + n_flex]).  placement is tagged in place."""
    assert counts.dtype == np.uint32
    R = counts.shape[0]
    cap = R if cap is None else cap
    rows = np.full(max(cap, 0) + 16, -1, dtype=np.int64)
    cuts = np.full(N_CUTS, -1, dtype=np.int64)
    tp = TierParams(**params)
    status = ctypes.c_int32(0)
    rc = lib().oracle_plan_tiers(_p(counts), ctypes.c_int64(R), ctypes.byref(tp), ctypes.c_int32(tiers), _p(rows),
                                 ctypes.c_int64(cap), _p(cuts), _p(placement), ctypes.byref(status))
    k = int(min(max(cuts[CUT_N_DP] + cuts[CUT_N_FLEX], 0), max(cap, 0))) if rc == 0 else 0
    assert np.all(rows[k:] == -1), "the oracle wrote past the rows it reports"
    return rc, cuts, rows[:k]


def sparse_update(weights: np.ndarray, uniq_rows, row_grads: np.ndarray, optimizer: int, lr: float, eps: float,
                  state: Optional[np.ndarray] = None, store: Optional[np.ndarray] = None, slot_of_row=None,
                  dtype: Optional[int] = None) -> Tuple[int, int]:
    """One optimizer step on the rows named by uniq_rows; weights, state and store change in place."""
    code = _dtype_code(weights, dtype)
    rows = _i64(uniq_rows)
    R, D = weights.shape
    assert row_grads.dtype == np.float32 and (state is None or state.dtype == np.float32)
    slots = None if slot_of_row is None else np.ascontiguousarray(slot_of_row, dtype=np.int32)
    k = 0 if store is None else store.shape[0]
    status = ctypes.c_int32(0)
    rc = lib().oracle_sparse_update(
        _p(weights), ctypes.c_int64(R), ctypes.c_int32(D), ctypes.c_int(code), _p(rows), _p(row_grads),
        ctypes.c_int64(rows.shape[0]), ctypes.c_int32(optimizer), ctypes.c_float(lr), ctypes.c_float(eps), _p(state),
        _p(store), _p(slots), ctypes.c_int64(k), ctypes.byref(status))
    return rc, status.value

"""CPU oracle (test infrastructure): ctypes view of oracle/agg_oracle.c.

Only tests, the smoke check and the bench's cpu_baseline leg may import this
package.  It imports nothing from the HIP path.  Arrays are numpy; bf16 data is
carried as uint16 bit patterns.  Each function mirrors one C routine; the
arithmetic is all in the C file.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

_LIB = None


def lib() -> C.CDLL:
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.oracle_f32_to_bf16.restype = C.c_uint16
        L.oracle_f32_to_bf16.argtypes = [C.c_float]
        L.oracle_bf16_to_f64.restype = C.c_double
        L.oracle_bf16_to_f64.argtypes = [C.c_uint16]
        L.oracle_threads.restype = C.c_int
        L.oracle_rs_required_bandwidth.restype = C.c_double
        L.oracle_rs_required_bandwidth.argtypes = [C.c_int, C.c_double, C.c_double]
        for name in ("oracle_allgather", "oracle_gemm", "oracle_ag_gemm", "oracle_rs_reduce_f64",
                     "oracle_rs_reduce_f32", "oracle_gemm_rs", "oracle_moe_route", "oracle_moe_gemm"):
            getattr(L, name).restype = C.c_int
        _LIB = L
    return _LIB


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("bf16 data must be uint16 bit patterns")
    return a


def _ptr(a: np.ndarray):
    return C.c_void_p(a.ctypes.data)


def _ptr_array(arrs):
    return (C.c_void_p * len(arrs))(*[a.ctypes.data if a is not None else None for a in arrs])


def _rows(rows):
    if rows is None:
        return None, C.c_void_p(None)
    r = np.ascontiguousarray(rows, dtype=np.int64)
    return r, _ptr(r)


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"{what}: oracle rejected the arguments (code {rc})")


def threads() -> int:
    return int(lib().oracle_threads())


def f32_to_bf16(x: float) -> int:
    return int(lib().oracle_f32_to_bf16(float(np.float32(x))))


def bf16_to_f64(bits: int) -> float:
    return float(lib().oracle_bf16_to_f64(int(bits)))


def allgather(shards, rank: int) -> np.ndarray:
    """Algorithm 2's gathered buffer T for `rank`: shard r at offset r*|L|. Returns [W*Ms, K] uint16."""
    shards = [_u16(s) for s in shards]
    W = len(shards)
    Ms, K = shards[0].shape
    T = np.empty((W * Ms, K), dtype=np.uint16)
    _check(lib().oracle_allgather(C.c_int(W), C.c_int(rank), C.c_int64(Ms * K), _ptr_array(shards), _ptr(T)),
           "allgather")
    return T


def gemm(A, B_kn, rows=None) -> np.ndarray:
    """fp64 C = A . B on bf16-bit inputs; A [M,K], B [K,N]. rows selects rows of A."""
    A = _u16(A)
    B = _u16(B_kn)
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    r, rp = _rows(rows)
    n = M if r is None else len(r)
    Cm = np.empty((n, N), dtype=np.float64)
    _check(lib().oracle_gemm(C.c_int64(M), C.c_int64(K), C.c_int64(N), _ptr(A), _ptr(B), rp, C.c_int64(n),
                             _ptr(Cm)), "gemm")
    return Cm


def ag_gemm(shards, B_kn, rank: int = 0, rows=None) -> np.ndarray:
    """fp64 C = gather(shards) . B for one rank; rows selects rows of the gathered matrix."""
    shards = [_u16(s) for s in shards]
    B = _u16(B_kn)
    W = len(shards)
    Ms, K = shards[0].shape
    K2, N = B.shape
    assert K == K2 and all(s.shape == (Ms, K) for s in shards)
    r, rp = _rows(rows)
    n = W * Ms if r is None else len(r)
    Cm = np.empty((n, N), dtype=np.float64)
    _check(lib().oracle_ag_gemm(C.c_int(W), C.c_int(rank), C.c_int64(Ms), C.c_int64(K), C.c_int64(N),
                                _ptr_array(shards), _ptr(B), rp, C.c_int64(n), _ptr(Cm)), "ag_gemm")
    return Cm


def _f32_slots(slots):
    out = []
    for s in slots:
        s = np.ascontiguousarray(s)
        if s.dtype != np.float32:
            raise TypeError("partial-sum slots must be float32")
        out.append(s)
    return out


def rs_reduce_f64(slots) -> np.ndarray:
    """fp64 sum of the W fp32 slots (definition of the reduction)."""
    slots = _f32_slots(slots)
    R = np.empty(slots[0].shape, dtype=np.float64)
    _check(lib().oracle_rs_reduce_f64(C.c_int(len(slots)), C.c_int64(slots[0].size), _ptr_array(slots), _ptr(R)),
           "rs_reduce_f64")
    return R


def rs_reduce_f32(slots) -> np.ndarray:
    """fp32 sum in the order w = 0..W-1 starting from +0 (Algorithm 3, stream 2)."""
    slots = _f32_slots(slots)
    R = np.empty(slots[0].shape, dtype=np.float32)
    _check(lib().oracle_rs_reduce_f32(C.c_int(len(slots)), C.c_int64(slots[0].size), _ptr_array(slots), _ptr(R)),
           "rs_reduce_f32")
    return R


def gemm_rs(A_loc, B_kn, peer_slots: dict, W: int, rank: int, rows=None) -> np.ndarray:
    """fp64 R = (A_loc . B_loc)[rank's row slice] + sum of the peers' fp32 slices."""
    A = _u16(A_loc)
    B = _u16(B_kn)
    M, Kl = A.shape
    K2, N = B.shape
    assert Kl == K2
    Ms = M // W
    arr = []
    for w in range(W):
        if w == rank:
            arr.append(None)
        else:
            s = np.ascontiguousarray(peer_slots[w])
            assert s.dtype == np.float32 and s.shape == (Ms, N)
            arr.append(s)
    r, rp = _rows(rows)
    n = Ms if r is None else len(r)
    R = np.empty((n, N), dtype=np.float64)
    _check(lib().oracle_gemm_rs(C.c_int(W), C.c_int(rank), C.c_int64(M), C.c_int64(Kl), C.c_int64(N),
                                _ptr(A), _ptr(B), _ptr_array(arr), rp, C.c_int64(n), _ptr(R)), "gemm_rs")
    return R


def moe_route(topk_ids, E: int):
    """(pair_token, pair_slot, seg_off): pairs sorted by (expert, token, slot)."""
    ids = np.ascontiguousarray(topk_ids, dtype=np.int32)
    T, topk = ids.shape
    tok = np.empty(T * topk, dtype=np.int32)
    slot = np.empty(T * topk, dtype=np.int32)
    seg = np.empty(E + 1, dtype=np.int64)
    _check(lib().oracle_moe_route(C.c_int64(T), C.c_int(topk), C.c_int(E), _ptr(ids), _ptr(tok), _ptr(slot),
                                  _ptr(seg)), "moe_route")
    return tok, slot, seg


def moe_gemm(shards, W_ekn, topk_ids, rank: int = 0, rows=None) -> np.ndarray:
    """fp64 Y[p, :] = X[token(p), :] . W_expert(p) over the sorted pair list."""
    shards = [_u16(s) for s in shards]
    Wt = _u16(W_ekn)
    ids = np.ascontiguousarray(topk_ids, dtype=np.int32)
    W = len(shards)
    tpr, K = shards[0].shape
    E, K2, N = Wt.shape
    assert K == K2
    T, topk = ids.shape
    assert T == W * tpr
    r, rp = _rows(rows)
    n = T * topk if r is None else len(r)
    Y = np.empty((n, N), dtype=np.float64)
    _check(lib().oracle_moe_gemm(C.c_int(W), C.c_int(rank), C.c_int64(tpr), C.c_int64(K), C.c_int64(N),
                                 C.c_int(E), C.c_int(topk), _ptr_array(shards), _ptr(Wt), _ptr(ids), rp,
                                 C.c_int64(n), _ptr(Y)), "moe_gemm")
    return Y


def moe_rs(H, W2_ekn, topk_ids, gate, peer_slots: dict, W: int, rank: int, rows=None) -> np.ndarray:
    """fp64 R for one rank: grouped GEMM on the routed rows H, top-k weighted reduction, plus the peers' slices."""
    H = _u16(H)
    W2 = _u16(W2_ekn)
    ids = np.ascontiguousarray(topk_ids, dtype=np.int32)
    g = np.ascontiguousarray(gate, dtype=np.float32)
    T, topk = ids.shape
    E, Kl, N = W2.shape
    assert H.shape == (T * topk, Kl) and g.shape == (T, topk) and T % W == 0
    Tr = T // W
    arr = []
    for w in range(W):
        if w == rank:
            arr.append(None)
        else:
            s_ = np.ascontiguousarray(peer_slots[w])
            assert s_.dtype == np.float32 and s_.shape == (Tr, N)
            arr.append(s_)
    r, rp = _rows(rows)
    n = Tr if r is None else len(r)
    R = np.empty((n, N), dtype=np.float64)
    _check(lib().oracle_moe_rs(C.c_int(W), C.c_int(rank), C.c_int64(T), C.c_int64(Kl), C.c_int64(N), C.c_int(E),
                               C.c_int(topk), _ptr(H), _ptr(W2), _ptr(ids), _ptr(g), _ptr_array(arr), rp, C.c_int64(n),
                               _ptr(R)), "moe_rs")
    return R


def rs_required_bandwidth(W: int, link_GBps: float, nic_GBps: float) -> float:
    return float(lib().oracle_rs_required_bandwidth(C.c_int(W), C.c_double(link_GBps), C.c_double(nic_GBps)))

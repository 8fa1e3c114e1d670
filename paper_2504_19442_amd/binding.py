"""ctypes binding with the names of include/agg.h.  Argument marshalling only.

Pointers may be given as integers (device addresses) or as objects with a
`data_ptr()` method (torch tensors); streams as integers (hipStream_t), objects
with a `cuda_stream` attribute (torch.cuda.Stream), or None for the default
stream.  A negative return code raises AggError.
"""
from __future__ import annotations

import ctypes as C
import os

__all__ = [
    "AggError", "Ctx", "symm_alloc", "signal_reset", "signal_set", "ag_producer_emulate", "ag_gemm",
    "rs_reduce", "gemm_rs", "gemm_rs_scatter", "ag_moe_gemm", "ag_moe_gemm_static", "agg_reserve_b_kn", "agg_reserve_moe", "moe_rs", "agg_autotune_ag_gemm", "agg_mfma_ceiling", "agg_status", "agg_strerror", "agg_device_info", "lib_path",
    "BF16", "F32", "B_NK", "B_KN", "PRODUCER_KERNEL", "PRODUCER_SDMA", "PRODUCER_LINKS", "PRODUCER_SKIP_LOCAL", "PRODUCER_LOCAL_LAST", "PRODUCER_NARROW",
    "ORDER_ROTATED", "ORDER_SUBCHUNK", "SIGNAL_STRIDE",
    "OK", "ERR_INVALID_ARG", "ERR_UNSUPPORTED_SHAPE", "ERR_MISALIGNED", "ERR_HIP", "ERR_TIMEOUT", "ERR_NOMEM", "ERR_NOT_FOUND", "ERR_IO", "ERR_NOT_RESERVED",
    "agg_tune_table_size", "agg_tune_table_clear", "agg_tune_table_put", "agg_tune_table_get", "agg_tune_table_save", "agg_tune_table_load",
    "agg_tune_table_apply", "TuneResult",
    "EXPORTS",
]

BF16, F32 = 0, 1
B_NK, B_KN = 0, 1
PRODUCER_KERNEL, PRODUCER_SDMA, PRODUCER_LINKS, PRODUCER_SKIP_LOCAL, PRODUCER_LOCAL_LAST, PRODUCER_NARROW = 0, 1, 2, 0x100, 0x200, 0x400
ORDER_ROTATED, ORDER_SUBCHUNK = 0, 1
SIGNAL_STRIDE = 32
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED_SHAPE, ERR_MISALIGNED, ERR_HIP, ERR_TIMEOUT, ERR_NOMEM = 0, -1, -2, -3, -4, -5, -6
ERR_NOT_FOUND, ERR_IO, ERR_NOT_RESERVED = -7, -8, -9

# every symbol include/agg.h declares
EXPORTS = [
    "symm_alloc", "symm_free", "symm_staging", "symm_signals", "symm_epoch", "symm_streams", "signal_reset", "signal_set",
    "agg_set_wait_limit_us", "agg_status", "ag_producer_emulate", "ag_gemm", "rs_reduce", "gemm_rs", "gemm_rs_scatter", "agg_autotune_ag_gemm", "agg_mfma_ceiling",
    "ag_moe_gemm", "ag_moe_gemm_static", "agg_reserve_b_kn", "agg_reserve_moe", "moe_rs", "agg_set_tile_config", "agg_set_device_epoch", "agg_set_tile_order", "agg_set_rs_chunks", "agg_set_rs_own_slice_last", "agg_tune_table_size", "agg_tune_table_clear", "agg_tune_table_put", "agg_tune_table_get", "agg_tune_table_save", "agg_tune_table_load", "agg_tune_table_apply", "agg_set_link_rate", "agg_set_local_shard", "agg_strerror", "agg_device_info",
]


def lib_path() -> str:
    """The built library, beside this file."""
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libagg.so")


_LIB = None


def _lib() -> C.CDLL:
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise RuntimeError(
                f"{path} is missing: build the HIP extension first (python -c 'import __graft_entry__ as g; g.build()'). "
                "There is no CPU fallback.")
        L = C.CDLL(path)
        vp, i32, i64, u64, sz = C.c_void_p, C.c_int, C.c_int64, C.c_uint64, C.c_size_t
        L.symm_alloc.argtypes = [C.POINTER(vp), i32, i32, sz, i32]
        L.symm_free.argtypes = [vp]
        L.symm_staging.argtypes = [vp]
        L.symm_staging.restype = vp
        L.symm_signals.argtypes = [vp]
        L.symm_signals.restype = vp
        L.symm_epoch.argtypes = [vp]
        L.symm_streams.argtypes = [vp, C.POINTER(vp), C.POINTER(vp)]
        L.signal_reset.argtypes = [vp, vp]
        L.signal_set.argtypes = [vp, i32, vp]
        L.agg_set_wait_limit_us.argtypes = [vp, u64]
        L.agg_set_tile_config.argtypes = [vp, i32]
        L.agg_set_tile_order.argtypes = [vp, i32]
        L.agg_set_device_epoch.argtypes = [vp, i32]
        L.agg_set_rs_chunks.argtypes = [vp, i32]
        L.agg_set_rs_own_slice_last.argtypes = [vp, i32]
        L.agg_set_local_shard.argtypes = [vp, vp]
        L.agg_set_link_rate.argtypes = [vp, C.c_double]
        L.agg_status.argtypes = [vp]
        L.ag_producer_emulate.argtypes = [vp, C.POINTER(vp), C.POINTER(i32), i32, i32, i32, vp]
        L.ag_gemm.argtypes = [vp, i32, i32, i32, vp, i32, i32, vp, i32, i32, vp]
        L.rs_reduce.argtypes = [vp, i32, i32, C.POINTER(vp), vp, i32, i32, i32, vp]
        L.gemm_rs.argtypes = [vp, i32, i32, i32, vp, i32, vp, i32, i32, C.POINTER(vp), vp, vp, i32, i32, vp, vp]
        L.gemm_rs_scatter.argtypes = [vp, i32, i32, i32, vp, i32, vp, i32, i32, C.POINTER(vp), vp, C.POINTER(vp), i32, vp]
        L.agg_tune_table_size.argtypes = []
        L.agg_tune_table_clear.argtypes = []
        L.agg_tune_table_put.argtypes = [i32, i32, i32, i32, vp]
        L.agg_tune_table_get.argtypes = [i32, i32, i32, i32, vp]
        L.agg_tune_table_save.argtypes = [C.c_char_p]
        L.agg_tune_table_load.argtypes = [C.c_char_p]
        L.agg_tune_table_apply.argtypes = [vp, i32, i32, i32]
        L.agg_autotune_ag_gemm.argtypes = [vp, i32, i32, i32, vp, i32, i32, vp, i32, i32, C.POINTER(vp), i32, i32, vp]
        L.agg_mfma_ceiling.argtypes = [vp, i32, i32, C.POINTER(C.c_double), vp]
        L.moe_rs.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, C.POINTER(vp), vp, vp, i32, i32, vp, vp]
        L.ag_moe_gemm.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, i32, i32, vp]
        L.ag_moe_gemm_static.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, i32, i32, vp]
        L.agg_reserve_b_kn.argtypes = [vp, i32, i32]
        L.agg_reserve_moe.argtypes = [vp, i32, i32, i32, i32]
        L.agg_strerror.argtypes = [i32]
        L.agg_strerror.restype = C.c_char_p
        L.agg_device_info.argtypes = [C.POINTER(i32), C.POINTER(i32)]
        for name in EXPORTS:
            if name not in ("symm_staging", "symm_signals", "agg_strerror"):
                getattr(L, name).restype = i32
        _LIB = L
    return _LIB


class AggError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {agg_strerror(code)} ({code})")


def agg_strerror(code: int) -> str:
    return _lib().agg_strerror(int(code)).decode()


def _check(rc: int, what: str) -> int:
    if rc < 0:
        raise AggError(rc, what)
    return rc


def _ptr(x) -> C.c_void_p:
    if x is None:
        return C.c_void_p(None)
    if hasattr(x, "data_ptr"):
        return C.c_void_p(x.data_ptr())
    return C.c_void_p(int(x))


def _stream(s) -> C.c_void_p:
    if s is None:
        return C.c_void_p(None)
    if hasattr(s, "cuda_stream"):
        return C.c_void_p(s.cuda_stream)
    return C.c_void_p(int(s))


def _ptr_array(items):
    return (C.c_void_p * len(items))(*[_ptr(i).value for i in items])


class Ctx:
    """Owner of one agg_ctx* (symmetric buffer T, signals S, epoch)."""

    def __init__(self, handle: int, world_size: int, rank: int, shard_bytes: int, n_signals: int):
        self.handle = C.c_void_p(handle)
        self.world_size, self.rank, self.shard_bytes, self.n_signals = world_size, rank, shard_bytes, n_signals

    @property
    def staging(self) -> int:
        return int(_lib().symm_staging(self.handle) or 0)

    @property
    def signals(self) -> int:
        return int(_lib().symm_signals(self.handle) or 0)

    def streams(self):
        """(producer_stream, consumer_stream) as integer hipStream_t handles owned by the context."""
        p, c = C.c_void_p(None), C.c_void_p(None)
        _check(_lib().symm_streams(self.handle, C.byref(p), C.byref(c)), "symm_streams")
        return int(p.value), int(c.value)

    @property
    def epoch(self) -> int:
        return _check(_lib().symm_epoch(self.handle), "symm_epoch")

    def set_wait_limit_us(self, us: int) -> None:
        _check(_lib().agg_set_wait_limit_us(self.handle, int(us)), "agg_set_wait_limit_us")

    def set_tile_config(self, cfg: int) -> None:
        _check(_lib().agg_set_tile_config(self.handle, int(cfg)), "agg_set_tile_config")

    def set_tile_order(self, order: int) -> None:
        _check(_lib().agg_set_tile_order(self.handle, int(order)), "agg_set_tile_order")

    def set_rs_own_slice_last(self, on: bool) -> None:
        _check(_lib().agg_set_rs_own_slice_last(self.handle, 1 if on else 0), "agg_set_rs_own_slice_last")

    def set_device_epoch(self, on: bool) -> None:
        _check(_lib().agg_set_device_epoch(self.handle, 1 if on else 0), "agg_set_device_epoch")

    def set_rs_chunks(self, chunks: int) -> None:
        _check(_lib().agg_set_rs_chunks(self.handle, int(chunks)), "agg_set_rs_chunks")

    def set_local_shard(self, local_shard) -> None:
        _check(_lib().agg_set_local_shard(self.handle, _ptr(local_shard)), "agg_set_local_shard")

    def set_link_rate(self, gigabytes_per_second: float) -> None:
        _check(_lib().agg_set_link_rate(self.handle, float(gigabytes_per_second)), "agg_set_link_rate")

    def free(self) -> None:
        if self.handle:
            _check(_lib().symm_free(self.handle), "symm_free")
            self.handle = C.c_void_p(None)

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.free()


def symm_alloc(world_size: int, rank: int, shard_bytes: int, n_signals: int | None = None) -> Ctx:
    n_signals = world_size if n_signals is None else n_signals
    h = C.c_void_p(None)
    _check(_lib().symm_alloc(C.byref(h), world_size, rank, shard_bytes, n_signals), "symm_alloc")
    return Ctx(h.value, world_size, rank, shard_bytes, n_signals)


def signal_reset(ctx: Ctx, stream=None) -> None:
    _check(_lib().signal_reset(ctx.handle, _stream(stream)), "signal_reset")


def signal_set(ctx: Ctx, index: int, stream=None) -> None:
    _check(_lib().signal_set(ctx.handle, int(index), _stream(stream)), "signal_set")


def agg_status(ctx: Ctx) -> int:
    """AGG_OK or ERR_TIMEOUT (not raised: a time-out is a reportable state)."""
    rc = _lib().agg_status(ctx.handle)
    if rc not in (OK, ERR_TIMEOUT):
        raise AggError(rc, "agg_status")
    return rc


def ag_producer_emulate(ctx: Ctx, remote_shards, arrival_order=None, mode: int = PRODUCER_KERNEL,
                        n_workgroups: int = 0, stream=None) -> None:
    ptrs = _ptr_array(remote_shards)
    if arrival_order is None:
        order, n = None, 0
    else:
        n = len(arrival_order)
        order = (C.c_int * max(n, 1))(*arrival_order)
    _check(_lib().ag_producer_emulate(ctx.handle, ptrs, order, n, mode, n_workgroups, _stream(stream)),
           "ag_producer_emulate")


def ag_gemm(ctx: Ctx, M: int, N: int, K: int, B, ldb: int, b_layout: int, Cout, ldc: int, c_dtype: int,
            stream=None) -> None:
    _check(_lib().ag_gemm(ctx.handle, M, N, K, _ptr(B), ldb, b_layout, _ptr(Cout), ldc, c_dtype, _stream(stream)),
           "ag_gemm")


def rs_reduce(ctx: Ctx, Ms: int, N: int, slots, R, ldr: int, r_dtype: int, n_workgroups: int = 0, stream=None) -> None:
    _check(_lib().rs_reduce(ctx.handle, Ms, N, _ptr_array(slots), _ptr(R), ldr, r_dtype, n_workgroups, _stream(stream)),
           "rs_reduce")


def gemm_rs(ctx: Ctx, M: int, N: int, Klocal: int, A_local, lda: int, B_local, ldb: int, b_layout: int, slots,
            P_other, R, ldr: int, r_dtype: int, gemm_stream=None, reduce_stream=None) -> None:
    _check(_lib().gemm_rs(ctx.handle, M, N, Klocal, _ptr(A_local), lda, _ptr(B_local), ldb, b_layout,
                          _ptr_array(slots), _ptr(P_other), _ptr(R), ldr, r_dtype, _stream(gemm_stream),
                          _stream(reduce_stream)), "gemm_rs")


def gemm_rs_scatter(ctx: Ctx, M: int, N: int, Klocal: int, A_local, lda: int, B_local, ldb: int, b_layout: int,
                    slice_dst, P_other, slice_signal, first_slice: int, gemm_stream=None) -> None:
    """slice_signal: list of W device addresses (int) of signal words, None entries allowed, or None."""
    sig = None if slice_signal is None else _ptr_array(slice_signal)
    _check(_lib().gemm_rs_scatter(ctx.handle, M, N, Klocal, _ptr(A_local), lda, _ptr(B_local), ldb, b_layout,
                                  _ptr_array(slice_dst), _ptr(P_other), sig, first_slice, _stream(gemm_stream)),
           "gemm_rs_scatter")


class TuneResult(C.Structure):
    _fields_ = [("tile_config", C.c_int), ("tile_order", C.c_int), ("producer_workgroups", C.c_int),
                ("configs_tried", C.c_int), ("best_ms", C.c_float)]


def agg_tune_table_size() -> int:
    return _check(_lib().agg_tune_table_size(), "agg_tune_table_size")


def agg_tune_table_clear() -> None:
    _check(_lib().agg_tune_table_clear(), "agg_tune_table_clear")


def agg_tune_table_put(world_size: int, M: int, N: int, K: int, entry: TuneResult) -> None:
    _check(_lib().agg_tune_table_put(world_size, M, N, K, C.byref(entry)), "agg_tune_table_put")


def agg_tune_table_get(world_size: int, M: int, N: int, K: int):
    """The entry, or None where the table has none."""
    res = TuneResult()
    rc = _lib().agg_tune_table_get(world_size, M, N, K, C.byref(res))
    if rc == ERR_NOT_FOUND:
        return None
    _check(rc, "agg_tune_table_get")
    return res


def agg_tune_table_save(path: str) -> None:
    _check(_lib().agg_tune_table_save(os.fsencode(path)), "agg_tune_table_save")


def agg_tune_table_load(path: str) -> int:
    """Merges the file into the table; returns the number of entries read."""
    return _check(_lib().agg_tune_table_load(os.fsencode(path)), "agg_tune_table_load")


def agg_tune_table_apply(ctx: Ctx, M: int, N: int, K: int) -> bool:
    """True if the context now carries the table's entry for this problem, False if there is none."""
    rc = _lib().agg_tune_table_apply(ctx.handle, M, N, K)
    if rc == ERR_NOT_FOUND:
        return False
    _check(rc, "agg_tune_table_apply")
    return True


def agg_autotune_ag_gemm(ctx: Ctx, M: int, N: int, K: int, B, ldb: int, b_layout: int, Cout, ldc: int, c_dtype: int,
                         remote_shards, producer_mode: int = PRODUCER_KERNEL, runs_per_config: int = 3) -> TuneResult:
    res = TuneResult()
    _check(_lib().agg_autotune_ag_gemm(ctx.handle, M, N, K, _ptr(B), ldb, b_layout, _ptr(Cout), ldc, c_dtype,
                                       _ptr_array(remote_shards), producer_mode, runs_per_config, C.byref(res)),
           "agg_autotune_ag_gemm")
    return res


def moe_rs(ctx: Ctx, Ttok: int, topk: int, E: int, N: int, Klocal: int, H, weights2, topk_ids, gate, Y, sorted_token,
           sorted_expert_offsets, pair_pos, slots, Z_other, R, ldr: int, r_dtype: int, gemm_stream=None,
           reduce_stream=None) -> None:
    _check(_lib().moe_rs(ctx.handle, Ttok, topk, E, N, Klocal, _ptr(H), _ptr(weights2), _ptr(topk_ids), _ptr(gate), _ptr(Y),
                         _ptr(sorted_token), _ptr(sorted_expert_offsets), _ptr(pair_pos), _ptr_array(slots), _ptr(Z_other),
                         _ptr(R), ldr, r_dtype, _stream(gemm_stream), _stream(reduce_stream)), "moe_rs")


def agg_mfma_ceiling(ctx: Ctx, iterations: int, constant_operands: bool = False, stream=None) -> float:
    """Enqueues the register-resident MFMA loop; returns the flop of the launch (the caller times it)."""
    flop = C.c_double(0.0)
    _check(_lib().agg_mfma_ceiling(ctx.handle, int(iterations), 1 if constant_operands else 0, C.byref(flop),
                                   _stream(stream)), "agg_mfma_ceiling")
    return flop.value


def ag_moe_gemm(ctx: Ctx, Ttok: int, topk: int, E: int, N: int, K: int, topk_ids, weights, sorted_token,
                sorted_expert_offsets, Y, ldy: int, y_dtype: int, stream=None) -> None:
    _check(_lib().ag_moe_gemm(ctx.handle, Ttok, topk, E, N, K, _ptr(topk_ids), _ptr(weights), _ptr(sorted_token),
                              _ptr(sorted_expert_offsets), _ptr(Y), ldy, y_dtype, _stream(stream)), "ag_moe_gemm")


def ag_moe_gemm_static(ctx: Ctx, Ttok: int, topk: int, E: int, N: int, K: int, topk_ids, weights, sorted_token,
                       sorted_expert_offsets, Y, ldy: int, y_dtype: int, stream=None) -> None:
    _check(_lib().ag_moe_gemm_static(ctx.handle, Ttok, topk, E, N, K, _ptr(topk_ids), _ptr(weights), _ptr(sorted_token),
                                     _ptr(sorted_expert_offsets), _ptr(Y), ldy, y_dtype, _stream(stream)),
           "ag_moe_gemm_static")


def agg_reserve_b_kn(ctx: Ctx, N: int, K: int) -> None:
    _check(_lib().agg_reserve_b_kn(ctx.handle, N, K), "agg_reserve_b_kn")


def agg_reserve_moe(ctx: Ctx, Ttok: int, topk: int, E: int, N: int) -> None:
    _check(_lib().agg_reserve_moe(ctx.handle, Ttok, topk, E, N), "agg_reserve_moe")


def agg_device_info():
    cu, khz = C.c_int(0), C.c_int(0)
    _check(_lib().agg_device_info(C.byref(cu), C.byref(khz)), "agg_device_info")
    return cu.value, khz.value

"""Device-side harness shared by the GPU tests, bench.py and the smoke run: device buffers for the seeded inputs and
one AllGather-GEMM problem set up on a context (torch is used for memory and streams only; no arithmetic of the method)."""
import numpy as np
import torch

import paper_2504_19442_amd as agg


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns -> torch.bfloat16 tensor on cuda:0 with the same bits."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()
    return t.view(torch.bfloat16)


def host_bits(t: torch.Tensor) -> np.ndarray:
    """torch.bfloat16 tensor -> uint16 bit patterns on the host."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


NAN_BITS = 0x7FC0  # bf16 quiet NaN: a tile that reads staging before its signal shows up as NaN


class AgGemmRun:
    """Device state of one AllGather-GEMM problem: 'remote' shard buffers, B in [N, K], a context."""

    def __init__(self, inp, rank: int, chunks_per_shard: int = 1):
        sh = inp.shape
        self.inp, self.sh, self.rank = inp, sh, rank
        self.remote = [dev_bf16(s) for s in inp.shards]                    # L_r of every rank
        self.B_nk = dev_bf16(np.ascontiguousarray(inp.B_kn.T))             # [N, K], K contiguous
        self.ctx = agg.symm_alloc(sh.W, rank, sh.Ms * sh.K * 2, sh.W * chunks_per_shard)
        self.staging = None
        # the context's own stream pair (separate hardware queues), wrapped so torch can query them
        ps, cs = self.ctx.streams()
        self.prod = torch.cuda.ExternalStream(ps)
        self.cons = torch.cuda.ExternalStream(cs)

    def poison(self):
        """Fill T with NaN patterns (through a torch view of the staging pointer made once)."""
        n = self.sh.W * self.sh.Ms * self.sh.K
        if self.staging is None:
            self.staging = _tensor_from_ptr(self.ctx.staging, n)
        self.staging.fill_(float("nan"))
        torch.cuda.synchronize()

    def run(self, order=None, out_dtype=agg.F32, mode=agg.PRODUCER_KERNEL, tile=None, poison=True,
            consumer_first=True, n_workgroups=0):
        sh = self.sh
        if poison:
            self.poison()
        if tile is not None:
            self.ctx.set_tile_config(tile)
        agg.signal_reset(self.ctx)
        C = torch.full((sh.M, sh.N), float("nan"), device="cuda",
                       dtype=torch.float32 if out_dtype == agg.F32 else torch.bfloat16)
        torch.cuda.synchronize()

        def consume():
            agg.ag_gemm(self.ctx, sh.M, sh.N, sh.K, self.B_nk, sh.K, agg.B_NK, C, sh.N, out_dtype, self.cons)

        def produce():
            agg.ag_producer_emulate(self.ctx, self.remote, order, mode, n_workgroups, self.prod)

        if consumer_first:
            consume(); produce()
        else:
            produce(); consume()
        torch.cuda.synchronize()
        st = agg.agg_status(self.ctx)
        assert st == agg.OK, agg.agg_strerror(st)
        return C

    def close(self):
        self.ctx.free()


def _tensor_from_ptr(ptr: int, n_bf16: int) -> torch.Tensor:
    """A torch.bfloat16 view of device memory the library owns (used only to poison T)."""
    import ctypes

    class _Holder:
        pass

    h = _Holder()
    h.__cuda_array_interface__ = {"shape": (n_bf16,), "typestr": "<i2", "data": (ptr, False), "version": 3}
    return torch.as_tensor(h, device="cuda").view(torch.bfloat16)

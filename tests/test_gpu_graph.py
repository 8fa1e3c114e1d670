"""A whole run of the overlapped function recorded in a HIP graph and replayed (the epoch kept on the device).

Every replay is a run with a fresh epoch: T and C are poisoned by eager work between the replays, the inputs are
changed in place, and every replay's result is compared bit for bit with what the same calls give outside a graph.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2504_19442_amd as agg
import workloads as wl
from harness import AgGemmRun

pytestmark = pytest.mark.gpu


def test_run_recorded_in_a_graph_replays_with_a_fresh_epoch_each_time():
    sh = wl.AgGemmShape("ag_graph", 19, 4, 256, 512, 448)
    inp = wl.make_ag_gemm(sh, a_dist=("int", 2), b_dist=("int", 2))
    want = oracle.ag_gemm(inp.shards, inp.B_kn, 1)
    run = AgGemmRun(inp, 1, chunks_per_shard=2)
    ctx = run.ctx
    try:
        ctx.set_wait_limit_us(500000)
        ctx.set_device_epoch(True)
        # outside a graph first (also sets up everything that is created on first use); the mode changes nothing here
        for consumer_first in (True, False):
            C0 = run.run(consumer_first=consumer_first).cpu().numpy()
            assert np.array_equal(C0.astype(np.float64), want)
        C = torch.full((sh.M, sh.N), float("nan"), device="cuda", dtype=torch.float32)
        s0 = torch.cuda.Stream()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s0, capture_error_mode="thread_local"):
            agg.signal_reset(ctx, s0)
            run.prod.wait_stream(s0)
            run.cons.wait_stream(s0)
            agg.ag_producer_emulate(ctx, run.remote, None, agg.PRODUCER_KERNEL, 0, run.prod)
            agg.ag_gemm(ctx, sh.M, sh.N, sh.K, run.B_nk, sh.K, agg.B_NK, C, sh.N, agg.F32, run.cons)
            s0.wait_stream(run.prod)
            s0.wait_stream(run.cons)
        torch.cuda.synchronize()
        assert np.isnan(C.cpu().numpy()).all()           # recording runs nothing
        sign = 1.0
        for k in range(6):
            run.poison()                                  # eager work between the replays: T and C hold NaN again
            C.fill_(float("nan"))
            if k in (2, 4):                               # the inputs change in place: a replay must read them anew
                for r in run.remote:
                    r.neg_()
                sign = -sign
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            st = agg.agg_status(ctx)
            assert st == agg.OK, (k, agg.agg_strerror(st))
            got = C.cpu().numpy()
            assert np.array_equal(got.astype(np.float64), sign * want), k
        # back on the host, the epoch goes on from where the device's count stands
        ctx.set_device_epoch(False)
        if sign < 0:
            for r in run.remote:
                r.neg_()
        assert np.array_equal(run.run().cpu().numpy().astype(np.float64), want)
    finally:
        run.close()


def test_gemm_rs_recorded_in_a_graph():
    """GEMM + ReduceScatter for one rank: reset, the peers' signals, the GEMM and the reducer in one graph."""
    from harness import dev_bf16
    sh = wl.RS_TINY
    rank = 2
    inp = wl.make_gemm_rs(sh, rank=rank)
    W, M, Ms, Kl, N = sh.W, sh.M, sh.Ms, sh.Kl, sh.N
    A = dev_bf16(inp.A_loc)
    B_nk = dev_bf16(np.ascontiguousarray(inp.B_kn.T))
    slots = [torch.full((Ms, N), float("nan"), device="cuda", dtype=torch.float32) for _ in range(W)]
    for w, s in inp.peer_slots.items():
        slots[w].copy_(torch.from_numpy(s))
    ctx = agg.symm_alloc(W, rank, 16, W * 2)
    try:
        ctx.set_wait_limit_us(500000)
        ctx.set_rs_chunks(2)
        ps, cs = ctx.streams()
        gs, rs_ = torch.cuda.ExternalStream(ps), torch.cuda.ExternalStream(cs)
        P = torch.empty((M, N), device="cuda", dtype=torch.float32)
        R = torch.full((Ms, N), float("nan"), device="cuda", dtype=torch.float32)

        def enqueue(origin):
            agg.signal_reset(ctx, origin)
            gs.wait_stream(origin)
            rs_.wait_stream(origin)
            for w in range(W):
                if w != rank:
                    for c in range(2):
                        agg.signal_set(ctx, w * 2 + c, rs_)
            agg.gemm_rs(ctx, M, N, Kl, A, Kl, B_nk, Kl, agg.B_NK, slots, P, R, N, agg.F32, gs, rs_)
            origin.wait_stream(gs)
            origin.wait_stream(rs_)

        # outside a graph, epoch on the host: the reference result of these very calls
        s0 = torch.cuda.Stream()
        with torch.cuda.stream(s0):
            enqueue(s0)
        torch.cuda.synchronize()
        assert agg.agg_status(ctx) == agg.OK
        ref = R.cpu().numpy().copy()
        want = oracle.gemm_rs(inp.A_loc, inp.B_kn, inp.peer_slots, W, rank)
        assert np.linalg.norm(ref - want) / np.linalg.norm(want) <= 1e-4

        ctx.set_device_epoch(True)
        with torch.cuda.stream(s0):
            enqueue(s0)                                   # once more eagerly, epoch on the device
        torch.cuda.synchronize()
        assert np.array_equal(R.cpu().numpy().view(np.uint32), ref.view(np.uint32))
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s0, capture_error_mode="thread_local"):
            enqueue(s0)
        for k in range(4):
            R.fill_(float("nan"))
            slots[rank].fill_(float("nan"))               # the own slot is produced anew by every replay
            P.fill_(float("nan"))
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            st = agg.agg_status(ctx)
            assert st == agg.OK, (k, agg.agg_strerror(st))
            assert np.array_equal(R.cpu().numpy().view(np.uint32), ref.view(np.uint32)), k
    finally:
        ctx.free()

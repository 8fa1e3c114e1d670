"""GPU parity of the ReduceScatter reducer and of GEMM-ReduceScatter against the CPU oracle, through the C ABI.

Bars: the reducer is bit-exact against the oracle's ordered fp32 sum (Algorithm 3, stream 2) whatever the order
in which the slots' signals are raised; GEMM-RS is within rel. Frobenius 1e-4 and max abs 1e-3*sqrt(K) of
the fp64 oracle, and bit-identical across signal orders.
"""
import itertools
import time

import numpy as np
import pytest
import torch

import oracle
import paper_2504_19442_amd as agg
import workloads as wl
from harness import dev_bf16, host_bits

pytestmark = pytest.mark.gpu


class RsRun:
    """W fp32 slots on the device (poisoned until they 'arrive'), a context and its stream pair."""

    def __init__(self, W, rank, Ms, N, n_signals=None):
        self.W, self.rank, self.Ms, self.N = W, rank, Ms, N
        self.ctx = agg.symm_alloc(W, rank, 16, n_signals or W)
        self.step = (n_signals or W) // W
        self.chunks = 1
        ps, cs = self.ctx.streams()
        self.prod = torch.cuda.ExternalStream(ps)
        self.cons = torch.cuda.ExternalStream(cs)
        self.slots = [torch.full((Ms, N), float("nan"), device="cuda", dtype=torch.float32) for _ in range(W)]

    def deliver(self, w, data, sleep=0.0):
        """Slot w arrives: its data lands (on the producer stream), then its signal is raised."""
        if sleep:
            time.sleep(sleep)
        with torch.cuda.stream(self.prod):
            self.slots[w].copy_(data, non_blocking=True)
        for c in range(self.chunks):
            agg.signal_set(self.ctx, w * self.step + c, self.prod)

    def set_chunks(self, chunks):
        """Slots arrive (and are waited for) in this many row chunks, each with its own signal."""
        self.chunks = chunks
        self.ctx.set_rs_chunks(chunks)

    def poison(self):
        for s in self.slots:
            s.fill_(float("nan"))
        torch.cuda.synchronize()

    def status_ok(self):
        torch.cuda.synchronize()
        st = agg.agg_status(self.ctx)
        assert st == agg.OK, agg.agg_strerror(st)

    def close(self):
        self.ctx.free()


def _slots_with_cancellation(W, Ms, N, seed):
    """fp32 slots whose sum depends on the order of the additions (mixed magnitudes and signs)."""
    rng = np.random.default_rng(seed)
    out = []
    for w in range(W):
        mag = np.float32(10.0) ** rng.integers(-3, 5, size=(Ms, N)).astype(np.float32)
        out.append((rng.standard_normal((Ms, N)).astype(np.float32) * mag).astype(np.float32))
    return out


@pytest.mark.parametrize("W,Ms,N", [(4, 64, 192), (8, 33, 100), (3, 7, 36), (1, 5, 8), (2, 130, 260), (5, 64, 64)])
def test_reducer_bit_exact_in_any_signal_order(W, Ms, N):
    data = _slots_with_cancellation(W, Ms, N, seed=7000 + W)
    want = oracle.rs_reduce_f32(data)
    # the order matters for these values: a reversed fp32 sum differs somewhere (the test would not see a wrong order otherwise)
    if W > 2:
        assert not np.array_equal(want, oracle.rs_reduce_f32(data[::-1]))
    dev = [torch.from_numpy(d).cuda() for d in data]
    run = RsRun(W, 0, Ms, N)
    try:
        orders = list(itertools.permutations(range(W)))
        rng = np.random.default_rng(1)
        picks = [orders[0], orders[-1]] + [orders[i] for i in rng.choice(len(orders), size=min(4, len(orders)), replace=False)]
        for k, order in enumerate(picks):
            run.poison()
            agg.signal_reset(run.ctx)
            R = torch.full((Ms, N), float("nan"), device="cuda", dtype=torch.float32)
            torch.cuda.synchronize()
            if k % 2 == 0:       # reducer launched first: it must wait for every slot
                agg.rs_reduce(run.ctx, Ms, N, run.slots, R, N, agg.F32, 0, run.cons)
                for w in order:
                    run.deliver(w, dev[w], sleep=0.002 if k == 0 else 0.0)
            else:
                for w in order:
                    run.deliver(w, dev[w])
                agg.rs_reduce(run.ctx, Ms, N, run.slots, R, N, agg.F32, 0, run.cons)
            run.status_ok()
            got = R.cpu().numpy()
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), f"order {order}"
    finally:
        run.close()


def test_reducer_bf16_output_strided_and_workgroup_counts():
    W, Ms, N = 4, 48, 72
    data = _slots_with_cancellation(W, Ms, N, seed=7100)
    want32 = oracle.rs_reduce_f32(data)
    want16 = wl.f32_to_bf16_bits(want32)
    dev = [torch.from_numpy(d).cuda() for d in data]
    run = RsRun(W, 2, Ms, N, n_signals=3 * W)     # several signals per shard: slot w uses the first of its group
    try:
        for nwg in (0, 1, 3, 1000):
            for dtype, ldr in ((agg.BF16, N), (agg.BF16, N + 8), (agg.F32, N + 4)):
                run.poison()
                agg.signal_reset(run.ctx)
                tdt = torch.bfloat16 if dtype == agg.BF16 else torch.float32
                R = torch.zeros((Ms, ldr), device="cuda", dtype=tdt)
                torch.cuda.synchronize()
                agg.rs_reduce(run.ctx, Ms, N, run.slots, R, ldr, dtype, nwg, run.cons)
                for w in (3, 1, 0, 2):
                    run.deliver(w, dev[w])
                run.status_ok()
                if dtype == agg.BF16:
                    got = host_bits(R)
                    assert np.array_equal(got[:, :N], want16)
                    assert not got[:, N:].any()                       # padding columns untouched
                else:
                    got = R.cpu().numpy()
                    assert np.array_equal(got[:, :N].view(np.uint32), want32.view(np.uint32))
                    assert not got[:, N:].any()
    finally:
        run.close()


def test_reducer_times_out_when_a_slot_never_arrives():
    W, Ms, N = 4, 16, 32
    run = RsRun(W, 0, Ms, N)
    try:
        run.ctx.set_wait_limit_us(20000)
        agg.signal_reset(run.ctx)
        R = torch.zeros((Ms, N), device="cuda", dtype=torch.float32)
        zero = torch.zeros((Ms, N), device="cuda", dtype=torch.float32)
        agg.rs_reduce(run.ctx, Ms, N, run.slots, R, N, agg.F32, 0, run.cons)
        for w in (0, 1, 3):                       # slot 2 never arrives
            run.deliver(w, zero)
        torch.cuda.synchronize()
        assert agg.agg_status(run.ctx) == agg.ERR_TIMEOUT
        assert agg.agg_status(run.ctx) == agg.OK  # the record is cleared by the first status call
    finally:
        run.close()


def test_reducer_argument_errors():
    run = RsRun(4, 0, 8, 8)
    try:
        R = torch.zeros((8, 8), device="cuda", dtype=torch.float32)
        with pytest.raises(agg.AggError):
            agg.rs_reduce(run.ctx, 8, 8, run.slots[:3] + [None], R, 8, agg.F32)       # a null slot
        with pytest.raises(agg.AggError):
            agg.rs_reduce(run.ctx, 8, 8, run.slots, R, 4, agg.F32)                    # ldr < N
        with pytest.raises(agg.AggError):
            agg.rs_reduce(run.ctx, 3, 3, run.slots, R, 3, agg.F32)                    # 9 elements: not a multiple of 4
        with pytest.raises(agg.AggError):
            agg.rs_reduce(run.ctx, 8, 8, run.slots, R, 8, 7)                          # unknown dtype
        agg.rs_reduce(run.ctx, 0, 8, run.slots, R, 8, agg.F32)                        # empty: a no-op
        run.status_ok()
    finally:
        run.close()


# ----------------------------------------------------------------------------------------------------------------
# GEMM + ReduceScatter
# ----------------------------------------------------------------------------------------------------------------

def _gemm_rs_case(shape, rank, rows_own, rows_other, tile=None, with_other=True, orders=1, chunks=1, own_last=False):
    inp = wl.make_gemm_rs(shape, rank=rank)
    W, M, Ms, Kl, N = shape.W, shape.M, shape.Ms, shape.Kl, shape.N
    A = dev_bf16(inp.A_loc)
    B_nk = dev_bf16(np.ascontiguousarray(inp.B_kn.T))
    peers = {w: torch.from_numpy(s).cuda() for w, s in inp.peer_slots.items()}
    run = RsRun(W, rank, Ms, N, n_signals=W * chunks)
    results = []
    try:
        if tile is not None:
            run.ctx.set_tile_config(tile)
        run.set_chunks(chunks)
        run.ctx.set_rs_own_slice_last(own_last)
        others = [w for w in range(W) if w != rank]
        rng = np.random.default_rng(11)
        for k in range(orders):
            order = others if k == 0 else list(rng.permutation(others))
            run.poison()
            agg.signal_reset(run.ctx)
            P = torch.full((M, N), float("nan"), device="cuda", dtype=torch.float32) if with_other else None
            R = torch.full((Ms, N), float("nan"), device="cuda", dtype=torch.float32)
            torch.cuda.synchronize()
            # the peers' partial sums arrive on the GEMM's stream: before the launch (odd runs) or after it (even runs);
            # the reducer, on the other stream, is launched before the late ones exist
            if k % 2 == 1:
                for w in order:
                    run.deliver(w, peers[w])
            agg.gemm_rs(run.ctx, M, N, Kl, A, Kl, B_nk, Kl, agg.B_NK, run.slots, P, R, N, agg.F32, run.prod, run.cons)
            if k % 2 == 0:
                for w in order:
                    run.deliver(w, peers[w])
            run.status_ok()
            results.append((R.cpu().numpy(), None if P is None else P))
        R0 = results[0][0]
        for Rk, _ in results[1:]:
            assert np.array_equal(Rk.view(np.uint32), R0.view(np.uint32))
        # own slice + peers against the fp64 oracle
        want = oracle.gemm_rs(inp.A_loc, inp.B_kn, inp.peer_slots, W, rank, rows=rows_own)
        got = R0[rows_own].astype(np.float64)
        rel = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30)
        assert rel <= 1e-4, rel
        assert np.abs(got - want).max() <= 1e-3 * np.sqrt(Kl)
        # the slot the GEMM wrote is exactly what the reducer added: R - peers (in order) is reproducible on the host
        own = run.slots[rank].cpu().numpy()
        ordered = [inp.peer_slots[w] if w != rank else own for w in range(W)]
        assert np.array_equal(oracle.rs_reduce_f32(ordered).view(np.uint32), R0.view(np.uint32))
        if with_other:
            P = results[0][1]
            rows_other = np.asarray(rows_other)
            wantP = oracle.gemm(inp.A_loc, inp.B_kn, rows=rows_other)
            gotP = P[torch.from_numpy(rows_other).cuda()].cpu().numpy().astype(np.float64)
            relP = np.linalg.norm(gotP - wantP) / max(np.linalg.norm(wantP), 1e-30)
            assert relP <= 1e-4, relP
            assert np.abs(gotP - wantP).max() <= 1e-3 * np.sqrt(Kl)
            # rows of the own slice are never written to P_other
            assert torch.isnan(P[rank * Ms:(rank + 1) * Ms]).all()
    finally:
        run.close()


@pytest.mark.parametrize("rank", [0, 1, 3])
@pytest.mark.parametrize("tile", list(range(8)))
def test_gemm_rs_tiny(rank, tile):
    sh = wl.RS_TINY
    rows_other = [r for r in range(sh.M) if not (rank * sh.Ms <= r < (rank + 1) * sh.Ms)]
    _gemm_rs_case(sh, rank, np.arange(sh.Ms), rows_other, tile=tile, orders=3)


def test_gemm_rs_own_slice_only():
    sh = wl.RS_TINY
    _gemm_rs_case(sh, 2, np.arange(sh.Ms), [], with_other=False, orders=2)


@pytest.mark.parametrize("chunks,with_other,own_last", [(2, True, False), (8, True, True), (4, False, True), (1, True, True)])
def test_gemm_rs_tiny_with_chunk_signals(chunks, with_other, own_last):
    sh = wl.RS_TINY
    rank = 1
    rows_other = [r for r in range(sh.M) if not (rank * sh.Ms <= r < (rank + 1) * sh.Ms)] if with_other else []
    _gemm_rs_case(sh, rank, np.arange(sh.Ms), rows_other, with_other=with_other, orders=3, chunks=chunks, own_last=own_last)


@pytest.mark.parametrize("chunks,own_last", [(1, False), (4, False), (4, True), (1, True)])
def test_gemm_rs_full_size(chunks, own_last):
    # every row of the own slice (all of R), and of the other slices one row out of every 128-row block (the smallest
    # tile height), so that every m-tile of the launch is compared with the oracle
    sh = wl.RS_FULL
    rank = 5
    rng = np.random.default_rng(5)
    rows_own = np.arange(sh.Ms)
    own = set(range(rank * sh.Ms, (rank + 1) * sh.Ms))
    rows_other = np.array([b + int(rng.integers(0, 128)) for b in range(0, sh.M, 128) if b not in own], dtype=np.int64)
    _gemm_rs_case(sh, rank, rows_own, rows_other, orders=2, chunks=chunks, own_last=own_last)


# ----------------------------------------------------------------------------------------------------------------
# Algorithm 3 end to end: W emulated ranks on one GPU, each scattering its partial slices into the others' slots
# ----------------------------------------------------------------------------------------------------------------

def _all_ranks_gemm_rs(shape, reducers_first, tile=None, rows=None, chunks=1):
    import dataclasses
    W, M, Ms, Kl, N = shape.W, shape.M, shape.Ms, shape.Kl, shape.N
    inputs = [wl.make_gemm_rs(dataclasses.replace(shape, cfg=shape.cfg + 20 + r), rank=r) for r in range(W)]
    A = [dev_bf16(i.A_loc) for i in inputs]
    B = [dev_bf16(np.ascontiguousarray(i.B_kn.T)) for i in inputs]
    ranks = [RsRun(W, r, Ms, N, n_signals=W * chunks) for r in range(W)]   # slots[r][w]: rank r's slot for peer w, poisoned
    R = [torch.full((Ms, N), float("nan"), device="cuda", dtype=torch.float32) for _ in range(W)]
    try:
        for rr in ranks:
            if tile is not None:
                rr.ctx.set_tile_config(tile)
            rr.ctx.set_rs_chunks(chunks)
            agg.signal_reset(rr.ctx)
        torch.cuda.synchronize()

        def reducers():
            for r, rr in enumerate(ranks):
                agg.rs_reduce(rr.ctx, Ms, N, rr.slots, R[r], N, agg.F32, 0, rr.cons)

        def gemms():
            for w, rw in enumerate(ranks):                     # rank w computes P_w and scatters slice r to rank r
                dst = [ranks[r].slots[w] for r in range(W)]
                sig = [ranks[r].ctx.signals + (w * ranks[r].step) * agg.SIGNAL_STRIDE * 4 for r in range(W)]
                # start with the slice of the next rank, the own slice last (it does not have to travel)
                agg.gemm_rs_scatter(rw.ctx, M, N, Kl, A[w], Kl, B[w], Kl, agg.B_NK, dst, None, sig, (w + 1) % W, rw.prod)

        if reducers_first:
            reducers(); gemms()
        else:
            gemms(); reducers()
        for rr in ranks:
            rr.status_ok()
        # each rank's result is the ordered fp32 sum of what landed in its slots, bit for bit ...
        for r, rr in enumerate(ranks):
            slots = [s.cpu().numpy() for s in rr.slots]
            assert not any(np.isnan(s).any() for s in slots)
            assert np.array_equal(oracle.rs_reduce_f32(slots).view(np.uint32), R[r].cpu().numpy().view(np.uint32))
        # ... and all of them together are one GEMM over the concatenated K (the definition of GEMM + ReduceScatter)
        A_cat = np.concatenate([i.A_loc for i in inputs], axis=1)
        B_cat = np.concatenate([i.B_kn for i in inputs], axis=0)
        got = torch.cat(R).cpu().numpy().astype(np.float64)
        rows = np.arange(M) if rows is None else rows
        want = oracle.gemm(A_cat, B_cat, rows=rows)
        g = got[rows]
        rel = np.linalg.norm(g - want) / np.linalg.norm(want)
        assert rel <= 1e-4, rel
        assert np.abs(g - want).max() <= 1e-3 * np.sqrt(W * Kl)
    finally:
        for rr in ranks:
            rr.close()


@pytest.mark.parametrize("tile", list(range(8)))
def test_all_ranks_on_one_gpu_tiny(tile):
    # The GEMMs are launched before the reducers: eight streams share the device's few hardware queues, and a GEMM
    # queued behind a reducer that waits for that very GEMM's signal could not start.
    _all_ranks_gemm_rs(wl.RS_TINY, reducers_first=False, tile=tile)


def test_all_ranks_on_one_gpu_medium():
    sh = wl.GemmRsShape("gemm_rs_medium", 13, 4, 2048, 512, 1024)
    rows = np.sort(np.random.default_rng(2).choice(sh.M, size=64, replace=False))
    _all_ranks_gemm_rs(sh, reducers_first=False, rows=rows)


@pytest.mark.parametrize("chunks,tile", [(2, 0), (2, 1), (4, 2), (16, 1)])
def test_all_ranks_with_chunk_signals_tiny(chunks, tile):
    # 64-row slices in chunks of 32, 16 or 4 rows: a tile of 128 or 256 rows completes chunks of several slices at once
    _all_ranks_gemm_rs(wl.RS_TINY, reducers_first=False, tile=tile, chunks=chunks)


@pytest.mark.parametrize("chunks", [2, 4])
def test_all_ranks_with_chunk_signals_medium(chunks):
    # 512-row slices in chunks of 256 and 128 rows (whole tiles) -- and every chunk's signal must have been raised
    sh = wl.GemmRsShape("gemm_rs_medium", 13, 4, 2048, 512, 1024)
    rows = np.sort(np.random.default_rng(3).choice(sh.M, size=64, replace=False))
    _all_ranks_gemm_rs(sh, reducers_first=False, rows=rows, chunks=chunks)


@pytest.mark.parametrize("W,Ms,N,chunks", [(4, 64, 192, 4), (8, 48, 100, 3), (3, 14, 36, 7), (2, 256, 1024, 16), (1, 6, 8, 2)])
def test_reducer_with_chunk_signals_bit_exact_in_any_order(W, Ms, N, chunks):
    # the slots arrive chunk by chunk in a shuffled order of (slot, chunk); the reducer, launched first, may only read
    # what has been signalled (everything else is NaN), and the sum is the same bit for bit as with whole slots
    data = _slots_with_cancellation(W, Ms, N, seed=7100 + W)
    want = oracle.rs_reduce_f32(data)
    dev = [torch.from_numpy(d).cuda() for d in data]
    run = RsRun(W, 0, Ms, N, n_signals=W * 16)
    cr = Ms // chunks
    try:
        run.ctx.set_rs_chunks(chunks)
        rng = np.random.default_rng(5)
        for k in range(3):
            run.poison()
            agg.signal_reset(run.ctx)
            R = torch.full((Ms, N), float("nan"), device="cuda", dtype=torch.float32)
            torch.cuda.synchronize()
            pairs = [(w, c) for w in range(W) for c in range(chunks)]
            rng.shuffle(pairs)
            if k < 2:
                agg.rs_reduce(run.ctx, Ms, N, run.slots, R, N, agg.F32, 0 if k == 0 else 3, run.cons)
            for w, c in pairs:
                if k == 0:
                    time.sleep(0.001)
                with torch.cuda.stream(run.prod):
                    run.slots[w][c * cr:(c + 1) * cr].copy_(dev[w][c * cr:(c + 1) * cr], non_blocking=True)
                agg.signal_set(run.ctx, w * run.step + c, run.prod)
            if k == 2:
                agg.rs_reduce(run.ctx, Ms, N, run.slots, R, N, agg.F32, 0, run.cons)
            run.status_ok()
            assert np.array_equal(R.cpu().numpy().view(np.uint32), want.view(np.uint32)), f"round {k}"
        # shapes the chunking cannot cut are refused, and so are chunk counts beyond the signals there are
        with pytest.raises(agg.AggError):
            run.ctx.set_rs_chunks(17)
        with pytest.raises(agg.AggError):
            run.ctx.set_rs_chunks(0)
        if Ms % 5:
            run.ctx.set_rs_chunks(5)
            with pytest.raises(agg.AggError):
                agg.rs_reduce(run.ctx, Ms, N, run.slots, R, N, agg.F32, 0, run.cons)
    finally:
        run.close()


def test_reducer_with_chunk_signals_times_out_on_a_missing_chunk():
    W, Ms, N, chunks = 2, 8, 16, 2
    run = RsRun(W, 0, Ms, N, n_signals=W * chunks)
    try:
        run.ctx.set_rs_chunks(chunks)
        run.ctx.set_wait_limit_us(20000)
        agg.signal_reset(run.ctx)
        R = torch.zeros((Ms, N), device="cuda", dtype=torch.float32)
        for s in (0, 1, 2):              # chunk 1 of slot 1 never arrives
            agg.signal_set(run.ctx, s, run.prod)
        agg.rs_reduce(run.ctx, Ms, N, run.slots, R, N, agg.F32, 0, run.cons)
        torch.cuda.synchronize()
        assert agg.agg_status(run.ctx) == agg.ERR_TIMEOUT
    finally:
        run.close()


def test_all_ranks_seeded_random_shapes_and_chunkings():
    # world size, chunk count, rows per chunk (smaller and larger than a tile, not powers of two), width and tile
    # shape drawn from a seeded generator: chunk counters and signals of every (slice, chunk) must come out right
    rng = np.random.default_rng(77)
    done = 0
    while done < 14:
        W = int(rng.choice([1, 2, 3, 4, 5, 8]))
        k = int(rng.choice([1, 2, 3, 5, 8, 16]))
        rows_per_chunk = int(rng.choice([1, 2, 6, 8, 32, 40, 64, 128]))
        Ms = k * rows_per_chunk
        N = int(rng.choice([4, 36, 100, 224, 260, 512]))
        if W * Ms > 2048 or (rows_per_chunk * N) % 4:
            continue
        Kl = 64 * int(rng.integers(1, 4))
        tile = int(rng.choice([-1, 0, 1, 2, 3]))
        sh = wl.GemmRsShape(f"rs_random_{done}", 60 + done, W, W * Ms, Kl, N)
        _all_ranks_gemm_rs(sh, reducers_first=False, tile=None if tile < 0 else tile, chunks=k)
        done += 1


@pytest.mark.parametrize("chunks", [1, 2])
def test_all_ranks_pull_mode(chunks):
    # Pull mode (Section 3.5 names both): every rank keeps its whole partial product P_w at home and only notifies;
    # rank r's reducer reads slice r of every P_w in place.  Same kernels, other pointers: no slice has a destination of
    # its own (all go to P_other = P_w), signal (r, w) is raised by rank w's GEMM, and the reducer's slots point into
    # the peers' P buffers.
    import dataclasses
    sh = wl.RS_TINY
    W, M, Ms, Kl, N = sh.W, sh.M, sh.Ms, sh.Kl, sh.N
    inputs = [wl.make_gemm_rs(dataclasses.replace(sh, cfg=sh.cfg + 40 + r), rank=r) for r in range(W)]
    A = [dev_bf16(i.A_loc) for i in inputs]
    B = [dev_bf16(np.ascontiguousarray(i.B_kn.T)) for i in inputs]
    ranks = [RsRun(W, r, Ms, N, n_signals=W * chunks) for r in range(W)]
    P = [torch.full((M, N), float("nan"), device="cuda", dtype=torch.float32) for _ in range(W)]
    R = [torch.full((Ms, N), float("nan"), device="cuda", dtype=torch.float32) for _ in range(W)]
    try:
        for rr in ranks:
            rr.set_chunks(chunks)
            agg.signal_reset(rr.ctx)
        torch.cuda.synchronize()
        for w, rw in enumerate(ranks):
            sig = [ranks[r].ctx.signals + (w * ranks[r].step) * agg.SIGNAL_STRIDE * 4 for r in range(W)]
            agg.gemm_rs_scatter(rw.ctx, M, N, Kl, A[w], Kl, B[w], Kl, agg.B_NK, [None] * W, P[w], sig, (w + 1) % W, rw.prod)
        for r, rr in enumerate(ranks):
            pulled = [P[w][r * Ms:(r + 1) * Ms] for w in range(W)]
            agg.rs_reduce(rr.ctx, Ms, N, pulled, R[r], N, agg.F32, 0, rr.cons)
        for rr in ranks:
            rr.status_ok()
        for r in range(W):
            parts = [P[w][r * Ms:(r + 1) * Ms].cpu().numpy() for w in range(W)]
            assert np.array_equal(oracle.rs_reduce_f32(parts).view(np.uint32), R[r].cpu().numpy().view(np.uint32))
        A_cat = np.concatenate([i.A_loc for i in inputs], axis=1)
        B_cat = np.concatenate([i.B_kn for i in inputs], axis=0)
        got = torch.cat(R).cpu().numpy().astype(np.float64)
        want = oracle.gemm(A_cat, B_cat)
        assert np.linalg.norm(got - want) / np.linalg.norm(want) <= 1e-4
        assert np.abs(got - want).max() <= 1e-3 * np.sqrt(W * Kl)
    finally:
        for rr in ranks:
            rr.close()


def test_gemm_rs_scatter_argument_errors():
    sh = wl.RS_TINY
    run = RsRun(sh.W, 0, sh.Ms, sh.N)
    try:
        inp = wl.make_gemm_rs(sh, rank=0)
        A, B = dev_bf16(inp.A_loc), dev_bf16(np.ascontiguousarray(inp.B_kn.T))
        good = dict(M=sh.M, N=sh.N, K=sh.Kl, dst=run.slots, P=None, sig=None, first=0)
        def call(**kw):
            a = dict(good); a.update(kw)
            agg.gemm_rs_scatter(run.ctx, a["M"], a["N"], a["K"], A, sh.Kl, B, sh.Kl, agg.B_NK, a["dst"], a["P"], a["sig"],
                                a["first"], run.prod)
        for bad in (dict(first=sh.W), dict(first=-1), dict(M=sh.M + 1), dict(dst=run.slots[:3] + [None]), dict(K=sh.Kl + 8)):
            with pytest.raises(agg.AggError):
                call(**bad)
        call(N=0)                       # empty: a no-op
        call()
        run.status_ok()
    finally:
        run.close()

"""GPU parity: the HIP AllGather-GEMM consumer against the CPU oracle, through the C ABI."""
import itertools
import time

import numpy as np
import pytest
import torch

import oracle
import paper_2504_19442_amd as agg
import workloads as wl
from harness import AgGemmRun, bits_to_f64, dev_bf16, host_bits

pytestmark = pytest.mark.gpu


def check_f32(C_gpu: np.ndarray, C_ref: np.ndarray, K: int):
    """The contract's bar: relative Frobenius error <= 1e-4 and max abs error <= 1e-3 * sqrt(K)."""
    assert np.all(np.isfinite(C_gpu)), "NaN/Inf in the output: a tile read staging before its signal, or was skipped"
    diff = C_gpu.astype(np.float64) - C_ref
    rel = np.linalg.norm(diff) / max(np.linalg.norm(C_ref), 1e-300)
    assert rel <= 1e-4, f"relative Frobenius error {rel}"
    assert np.max(np.abs(diff)) <= 1e-3 * np.sqrt(K), f"max abs error {np.max(np.abs(diff))}"


def check_bf16(C_bits: np.ndarray, C_f32: np.ndarray, C_ref: np.ndarray, K: int):
    """bf16 output = RNE(fp32 accumulator) exactly; and within half a bf16 ulp (+ the fp32 bar) of the oracle."""
    want = torch.from_numpy(C_f32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(C_bits, want)
    got = bits_to_f64(C_bits)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(C_ref), 1e-30))) - 7)
    assert np.all(np.abs(got - C_ref) <= 0.5 * ulp + 1e-3 * np.sqrt(K) * 2.0**-8 + 1e-30)


@pytest.mark.parametrize("rank", [0, 1, 3])
def test_tiny_random_arrival_order(rank):
    inp = wl.make_ag_gemm(wl.AG_TINY)
    ref = oracle.ag_gemm(inp.shards, inp.B_kn, rank)
    run = AgGemmRun(inp, rank)
    try:
        rng = np.random.default_rng(1000 + rank)
        order = [int(x) for x in rng.permutation([r for r in range(inp.shape.W) if r != rank])]
        C = run.run(order).cpu().numpy()
        check_f32(C, ref, inp.shape.K)
    finally:
        run.close()


def test_tiny_bit_identical_over_all_arrival_orders_and_launch_orders():
    inp = wl.make_ag_gemm(wl.AG_TINY)
    run = AgGemmRun(inp, 0)
    try:
        base = None
        for order in itertools.permutations([1, 2, 3]):
            for consumer_first in (True, False):
                C = run.run(list(order), consumer_first=consumer_first).cpu().numpy()
                if base is None:
                    base = C
                    check_f32(C, oracle.ag_gemm(inp.shards, inp.B_kn, 0), inp.shape.K)
                assert np.array_equal(C.view(np.uint32), base.view(np.uint32)), f"order {order} changed the bits"
    finally:
        run.close()


@pytest.mark.parametrize("tile", list(range(8)))
def test_integer_inputs_are_exact(tile):
    # entries in {-2..2}: every partial sum is an integer below 2^24, so fp32 accumulation is exact
    inp = wl.make_ag_gemm(wl.AG_RAGGED, a_dist=("int", 2), b_dist=("int", 2))
    ref = oracle.ag_gemm(inp.shards, inp.B_kn, 1)
    run = AgGemmRun(inp, 1)
    try:
        C = run.run(tile=tile).cpu().numpy()
        assert np.array_equal(C.astype(np.float64), ref)
    finally:
        run.close()


def test_identity_b_returns_gathered_a_bit_exactly():
    sh = wl.AgGemmShape("eye", 9, 4, 64, 256, 256, out="f32")
    inp = wl.make_ag_gemm(sh)
    inp.B_kn = wl.f32_to_bf16_bits(np.eye(sh.K, dtype=np.float32))
    run = AgGemmRun(inp, 2)
    try:
        C = run.run(out_dtype=agg.BF16)
        assert np.array_equal(host_bits(C), np.concatenate(inp.shards))
    finally:
        run.close()


@pytest.mark.parametrize("tile", list(range(8)))
@pytest.mark.parametrize("chunks", [1, 4])
def test_ragged_shape_f32_and_bf16(tile, chunks):
    inp = wl.make_ag_gemm(wl.AG_RAGGED)         # M=600, N=328, K=320: ragged against every tile shape
    ref = oracle.ag_gemm(inp.shards, inp.B_kn, 2)
    run = AgGemmRun(inp, 2, chunks_per_shard=chunks)
    try:
        C32 = run.run(tile=tile).cpu().numpy()
        check_f32(C32, ref, inp.shape.K)
        C16 = host_bits(run.run(out_dtype=agg.BF16, tile=tile))
        check_bf16(C16, C32, ref, inp.shape.K)
    finally:
        run.close()


def test_shards_delivered_one_by_one_with_host_delays():
    # the consumer is launched first and must block on each shard until the host lets it arrive
    inp = wl.make_ag_gemm(wl.AG_TINY)
    sh = inp.shape
    ref = oracle.ag_gemm(inp.shards, inp.B_kn, 0)
    run = AgGemmRun(inp, 0)
    try:
        run.poison()
        agg.signal_reset(run.ctx)
        C = torch.full((sh.M, sh.N), float("nan"), device="cuda", dtype=torch.float32)
        torch.cuda.synchronize()
        agg.ag_gemm(run.ctx, sh.M, sh.N, sh.K, run.B_nk, sh.K, agg.B_NK, C, sh.N, agg.F32, run.cons)
        agg.ag_producer_emulate(run.ctx, run.remote, [], agg.PRODUCER_KERNEL, 4, run.prod)      # local only
        for r in (3, 1, 2):
            time.sleep(0.02)
            assert not run.cons.query(), "the consumer finished before every shard had arrived"
            agg.ag_producer_emulate(run.ctx, run.remote, [r], agg.PRODUCER_KERNEL | agg.PRODUCER_SKIP_LOCAL, 4,
                                    run.prod)
        torch.cuda.synchronize()
        assert agg.agg_status(run.ctx) == agg.OK
        check_f32(C.cpu().numpy(), ref, sh.K)
    finally:
        run.close()


def test_new_shard_contents_in_the_next_epoch_are_seen_without_any_poison_between():
    """Two runs on one context with different shard contents and nothing written to T in between: the second run's
    tiles must read what arrived in their own epoch, not lines a CU or an L2 kept from the first (the acquire after
    the wait is what guarantees it)."""
    inp1 = wl.make_ag_gemm(wl.AG_RAGGED)
    inp2 = wl.make_ag_gemm(wl.AG_RAGGED, a_dist=("int", 2))
    run = AgGemmRun(inp1, 1, chunks_per_shard=2)
    try:
        for tile in (0, 1):
            C1 = run.run(tile=tile, poison=False).cpu().numpy()
            check_f32(C1, oracle.ag_gemm(inp1.shards, inp1.B_kn, 1), inp1.shape.K)
            saved = [r.clone() for r in run.remote]
            for r, s in zip(run.remote, inp2.shards):           # new contents in the peers' buffers, same addresses
                r.copy_(dev_bf16(s))
            C2 = run.run([0, 2], tile=tile, poison=False, consumer_first=True).cpu().numpy()
            check_f32(C2, oracle.ag_gemm(inp2.shards, inp1.B_kn, 1), inp1.shape.K)
            for r, s in zip(run.remote, saved):
                r.copy_(s)
    finally:
        run.close()


def test_narrow_producer_delivers_the_same_bytes():
    """The copy kernel with workgroups of one wave (AGG_PRODUCER_NARROW): T ends up byte for byte the gathered shards and
    the product is bit-identical to the run with the four-wave producer, for whole and ragged chunk sizes."""
    for shape, chunks in ((wl.AG_TINY, 2), (wl.AG_RAGGED, 1), (wl.AG_8B, 4)):
        inp = wl.make_ag_gemm(shape)
        run = AgGemmRun(inp, 1, chunks_per_shard=chunks)
        try:
            base = run.run(consumer_first=False)
            for nwg in (0, 3, 37):
                C = run.run([0] + list(range(2, shape.W)), mode=agg.PRODUCER_KERNEL | agg.PRODUCER_NARROW,
                            n_workgroups=nwg)
                assert torch.equal(C.view(torch.int32), base.view(torch.int32)), (shape.name, nwg)
                n = shape.W * shape.Ms * shape.K
                from harness import _tensor_from_ptr
                T = _tensor_from_ptr(run.ctx.staging, n).view(torch.int16).cpu().numpy().view(np.uint16)
                assert np.array_equal(T.reshape(shape.M, shape.K), np.concatenate(inp.shards))
        finally:
            run.close()


def test_copy_engine_producer():
    inp = wl.make_ag_gemm(wl.AG_TINY)
    ref = oracle.ag_gemm(inp.shards, inp.B_kn, 1)
    run = AgGemmRun(inp, 1, chunks_per_shard=2)
    try:
        for _ in range(2):          # twice: the second run must not see the first run's signals or data
            C = run.run([0, 3, 2], mode=agg.PRODUCER_SDMA).cpu().numpy()
            check_f32(C, ref, inp.shape.K)
    finally:
        run.close()


def test_missing_shard_times_out_and_reports():
    inp = wl.make_ag_gemm(wl.AG_TINY)
    sh = inp.shape
    run = AgGemmRun(inp, 0)
    try:
        run.ctx.set_wait_limit_us(20000)         # the host never delivers shard 2: the wait is bounded
        agg.signal_reset(run.ctx)
        C = torch.zeros((sh.M, sh.N), device="cuda", dtype=torch.float32)
        agg.ag_producer_emulate(run.ctx, run.remote, [1, 3], agg.PRODUCER_KERNEL, 4, run.prod)
        agg.ag_gemm(run.ctx, sh.M, sh.N, sh.K, run.B_nk, sh.K, agg.B_NK, C, sh.N, agg.F32, run.cons)
        torch.cuda.synchronize()
        assert agg.agg_status(run.ctx) == agg.ERR_TIMEOUT
        assert agg.agg_status(run.ctx) == agg.OK      # the record is cleared
        # and the context still works afterwards
        run.ctx.set_wait_limit_us(2000000)
        C2 = run.run().cpu().numpy()
        check_f32(C2, oracle.ag_gemm(inp.shards, inp.B_kn, 0), sh.K)
    finally:
        run.close()


def test_argument_errors():
    inp = wl.make_ag_gemm(wl.AG_TINY)
    sh = inp.shape
    run = AgGemmRun(inp, 0)
    try:
        C = torch.zeros((sh.M, sh.N), device="cuda", dtype=torch.float32)
        def rc(**kw):
            a = dict(M=sh.M, N=sh.N, K=sh.K, B=run.B_nk, ldb=sh.K, b_layout=agg.B_NK, Cout=C, ldc=sh.N, c_dtype=agg.F32)
            a.update(kw)
            with pytest.raises(agg.AggError) as e:
                agg.ag_gemm(run.ctx, a["M"], a["N"], a["K"], a["B"], a["ldb"], a["b_layout"], a["Cout"], a["ldc"],
                            a["c_dtype"], None)
            return e.value.code
        assert rc(K=sh.K - 16) == agg.ERR_UNSUPPORTED_SHAPE
        assert rc(M=sh.M + 1) == agg.ERR_UNSUPPORTED_SHAPE
        assert rc(M=sh.M + 4) == agg.ERR_UNSUPPORTED_SHAPE          # shard size no longer matches T
        assert rc(B=None) == agg.ERR_INVALID_ARG
        assert rc(B=run.B_nk.data_ptr() + 2) == agg.ERR_MISALIGNED
        assert rc(ldb=sh.K + 4) == agg.ERR_MISALIGNED
        assert rc(ldc=sh.N - 1) == agg.ERR_INVALID_ARG
        assert rc(c_dtype=7) == agg.ERR_INVALID_ARG
        agg.ag_gemm(run.ctx, 0, sh.N, sh.K, run.B_nk, sh.K, agg.B_NK, C, sh.N, agg.F32, None)   # empty: no-op
        with pytest.raises(agg.AggError):
            agg.ag_producer_emulate(run.ctx, run.remote, [0], agg.PRODUCER_KERNEL, 0, None)    # own rank listed
        with pytest.raises(agg.AggError):
            agg.ag_producer_emulate(run.ctx, run.remote, [1, 1], agg.PRODUCER_KERNEL, 0, None)  # repeated
        torch.cuda.synchronize()
    finally:
        run.close()


# --------------------------------------------------------------------------- full-size workloads


@pytest.mark.parametrize("shape", [wl.AG_8B, wl.AG_70B])
def test_full_size_whole_matrix_and_order_invariance(shape):
    """The whole fp32 result against the oracle, element by element (every tile of the launch is compared, not a
    sample of rows), the bf16 result against both, and bit-identical outputs over 16 arrival orders."""
    inp = wl.make_ag_gemm(shape)
    rank = 3
    ref = oracle.ag_gemm(inp.shards, inp.B_kn, rank)           # all M rows: about 2 s (8B shape), 15-30 s (70B shape)
    run = AgGemmRun(inp, rank, chunks_per_shard=4)
    try:
        C32 = run.run(consumer_first=False).cpu().numpy()
        check_f32(C32, ref, shape.K)
        orders = wl.arrival_orders(shape.W, rank, limit=16, seed=shape.cfg)
        assert len(orders) >= 16
        base16 = None
        for order in orders:
            C16 = run.run(order, out_dtype=agg.BF16, consumer_first=False)
            if base16 is None:
                base16 = C16
                check_bf16(host_bits(C16), C32, ref, shape.K)   # = RNE(fp32 path) everywhere, and within the bf16 bar
            else:
                assert torch.equal(C16.view(torch.int16), base16.view(torch.int16)), \
                    f"arrival order {order} changed the output bits"
        # the configuration the benchmark times: own shard read in place, its copy into T last, producer launched first
        run.ctx.set_local_shard(run.remote[rank])
        C16 = run.run(None, out_dtype=agg.BF16, mode=agg.PRODUCER_KERNEL | agg.PRODUCER_LOCAL_LAST, consumer_first=False)
        assert torch.equal(C16.view(torch.int16), base16.view(torch.int16))
    finally:
        run.close()


# ----------------------------------------------------------------------------------------------------------------
# Full-mesh arrival (every peer on a link of its own, chunk by chunk) and the sub-chunk tile order (Section 3.7)
# ----------------------------------------------------------------------------------------------------------------

MESH_SHAPE = wl.AgGemmShape("ag_mesh_small", 10, 4, 256, 128, 256)


@pytest.mark.parametrize("rank", [0, 3])
def test_full_mesh_producer_and_subchunk_order_match_the_plain_run_bit_for_bit(rank):
    inp = wl.make_ag_gemm(MESH_SHAPE)
    want = oracle.ag_gemm(inp.shards, inp.B_kn, rank)
    run = AgGemmRun(inp, rank, chunks_per_shard=2)
    try:
        base = run.run(tile=1).cpu().numpy()                       # rotated order, shard-after-shard producer
        got64 = base.astype(np.float64)
        assert np.linalg.norm(got64 - want) / np.linalg.norm(want) <= 1e-4
        assert np.abs(got64 - want).max() <= 1e-3 * np.sqrt(MESH_SHAPE.K)
        for order in (agg.ORDER_SUBCHUNK, agg.ORDER_ROTATED):
            for rate in (0.0, 2.0):                                 # unpaced; 2 GB/s: a 64 KiB shard takes 32 us
                for tile in (1, 0):                                 # 128-row tiles walk sub-chunks; 256-row tiles cannot
                    run.ctx.set_tile_order(order)
                    run.ctx.set_link_rate(rate)
                    C = run.run(tile=tile, mode=agg.PRODUCER_LINKS, consumer_first=(tile == 1)).cpu().numpy()
                    if tile == 1:
                        assert np.array_equal(C.view(np.uint32), base.view(np.uint32)), (order, rate)
                    else:
                        assert np.abs(C.astype(np.float64) - want).max() <= 1e-3 * np.sqrt(MESH_SHAPE.K)
        # a subset of the peers, listed in any order: the others never arrive and the consumer reports it
        run.ctx.set_wait_limit_us(20000)
        run.ctx.set_tile_order(agg.ORDER_SUBCHUNK)
        run.poison()
        agg.signal_reset(run.ctx)
        C = torch.zeros((MESH_SHAPE.M, MESH_SHAPE.N), device="cuda", dtype=torch.float32)
        peers = [(rank + j) % MESH_SHAPE.W for j in (3, 1)]
        agg.ag_producer_emulate(run.ctx, run.remote, peers, agg.PRODUCER_LINKS, 0, run.prod)
        agg.ag_gemm(run.ctx, MESH_SHAPE.M, MESH_SHAPE.N, MESH_SHAPE.K, run.B_nk, MESH_SHAPE.K, agg.B_NK, C,
                    MESH_SHAPE.N, agg.F32, run.cons)
        torch.cuda.synchronize()
        assert agg.agg_status(run.ctx) == agg.ERR_TIMEOUT
    finally:
        run.close()


def test_paced_links_deliver_at_the_link_rate():
    sh = wl.AG_8B                                                   # 4 MiB shards
    inp = wl.make_ag_gemm(sh)
    run = AgGemmRun(inp, 2, chunks_per_shard=4)
    try:
        rate = 40.0                                                 # GB/s per link: 4 MiB take 104.9 us
        run.ctx.set_link_rate(rate)
        expect_ms = sh.Ms * sh.K * 2 / (rate * 1e9) * 1e3
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        times = []
        for _ in range(3):
            agg.signal_reset(run.ctx)
            e0.record(run.prod)
            agg.ag_producer_emulate(run.ctx, run.remote, None, agg.PRODUCER_LINKS, 0, run.prod)
            e1.record(run.prod)
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1))
        assert agg.agg_status(run.ctx) == agg.OK
        t = min(times)
        assert 0.95 * expect_ms <= t <= 3.0 * expect_ms, (t, expect_ms)      # never faster than the link
        # and the data is all there
        T = run.ctx.staging
        from harness import _tensor_from_ptr
        got = host_bits(_tensor_from_ptr(T, sh.W * sh.Ms * sh.K)).reshape(sh.M, sh.K)
        assert np.array_equal(got, np.concatenate(inp.shards))
    finally:
        run.close()


def test_full_size_full_mesh_paced_subchunk_order():
    sh = wl.AG_70B
    inp = wl.make_ag_gemm(sh)
    rank = 5
    run = AgGemmRun(inp, rank, chunks_per_shard=4)
    try:
        base = run.run(out_dtype=agg.BF16, consumer_first=False)
        run.ctx.set_tile_order(agg.ORDER_SUBCHUNK)
        run.ctx.set_link_rate(76.8)
        C = run.run(out_dtype=agg.BF16, mode=agg.PRODUCER_LINKS, consumer_first=True)
        assert torch.equal(C.view(torch.int16), base.view(torch.int16))
        rows = np.sort(np.random.default_rng(3).choice(sh.M, size=8, replace=False))
        want = oracle.ag_gemm(inp.shards, inp.B_kn, rank, rows=rows)
        got = bits_to_f64(host_bits(C[torch.from_numpy(rows).cuda()]))
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 1e-30))) - 7)
        assert np.all(np.abs(got - want) <= 0.5 * ulp + 1e-3 * np.sqrt(sh.K) * 2.0 ** -8)
    finally:
        run.close()


def test_world_of_one_is_a_plain_gemm():
    sh = wl.AgGemmShape("ag_w1", 12, 1, 200, 192, 136)
    inp = wl.make_ag_gemm(sh)
    want = oracle.gemm(inp.shards[0], inp.B_kn)
    assert np.array_equal(want, oracle.ag_gemm(inp.shards, inp.B_kn, 0))
    run = AgGemmRun(inp, 0)
    try:
        for tile in range(8):
            check_f32(run.run(tile=tile).cpu().numpy(), want, sh.K)
    finally:
        run.close()


@pytest.mark.parametrize("rank", [0, 2])
def test_own_shard_read_in_place(rank):
    """With agg_set_local_shard the consumer never touches the own shard's part of T: it may arrive last, or never."""
    inp = wl.make_ag_gemm(MESH_SHAPE)
    run = AgGemmRun(inp, rank, chunks_per_shard=2)
    sh = MESH_SHAPE
    try:
        base = run.run(tile=1).cpu().numpy()
        run.ctx.set_local_shard(run.remote[rank])
        for tile in (1, 0):
            ref = base if tile == 1 else run_plain(run, tile)
            for mode in (agg.PRODUCER_KERNEL, agg.PRODUCER_LINKS, agg.PRODUCER_SDMA):
                C = run.run(tile=tile, mode=mode | agg.PRODUCER_LOCAL_LAST).cpu().numpy()
                assert np.array_equal(C.view(np.uint32), ref.view(np.uint32)), (tile, mode)
                # T is complete afterwards all the same
                from harness import _tensor_from_ptr
                got = host_bits(_tensor_from_ptr(run.ctx.staging, sh.M * sh.K)).reshape(sh.M, sh.K)
                assert np.array_equal(got, np.concatenate(inp.shards))
            # the own shard never copied at all: its part of T stays poisoned, the result is still right
            C = run.run(tile=tile, mode=agg.PRODUCER_KERNEL | agg.PRODUCER_SKIP_LOCAL).cpu().numpy()
            assert np.array_equal(C.view(np.uint32), ref.view(np.uint32))
    finally:
        run.close()


def run_plain(run, tile):
    run.ctx.set_local_shard(None)
    out = run.run(tile=tile).cpu().numpy()
    run.ctx.set_local_shard(run.remote[run.rank])
    return out


def test_autotuner_runs_the_whole_function_and_leaves_a_working_configuration():
    inp = wl.make_ag_gemm(MESH_SHAPE)
    sh = MESH_SHAPE
    want = oracle.ag_gemm(inp.shards, inp.B_kn, 1)
    run = AgGemmRun(inp, 1, chunks_per_shard=2)
    try:
        C = torch.zeros((sh.M, sh.N), device="cuda", dtype=torch.float32)
        e_before = run.ctx.epoch
        res = agg.agg_autotune_ag_gemm(run.ctx, sh.M, sh.N, sh.K, run.B_nk, sh.K, agg.B_NK, C, sh.N, agg.F32, run.remote,
                                       agg.PRODUCER_KERNEL, 2)
        assert res.configs_tried == 24 and res.tile_config in (4, 5, 6, 7) and res.tile_order in (0, 1)
        assert res.producer_workgroups > 0 and 0.0 < res.best_ms < 1000.0
        assert run.ctx.epoch == e_before + 24 * 3 + 29     # the signals were reset before every single run
        check_f32(C.cpu().numpy(), want, sh.K)              # the last tuning run left a complete, correct C
        check_f32(run.run().cpu().numpy(), want, sh.K)      # and the chosen configuration works
        res2 = agg.agg_autotune_ag_gemm(run.ctx, sh.M, sh.N, sh.K, run.B_nk, sh.K, agg.B_NK, C, sh.N, agg.F32, run.remote,
                                        agg.PRODUCER_SDMA, 1)
        assert res2.configs_tried == 8 and res2.producer_workgroups == 0
        with pytest.raises(agg.AggError):
            agg.agg_autotune_ag_gemm(run.ctx, sh.M, sh.N, sh.K + 8, run.B_nk, sh.K, agg.B_NK, C, sh.N, agg.F32, run.remote,
                                     agg.PRODUCER_KERNEL, 1)
        # the tuner's results are kept: the table holds the latest one for this problem, and a new context takes it over
        ent = agg.agg_tune_table_get(sh.W, sh.M, sh.N, sh.K)
        assert (ent.tile_config, ent.tile_order, ent.producer_workgroups) == (res2.tile_config, res2.tile_order, 0)
        other = AgGemmRun(inp, 1, chunks_per_shard=2)
        try:
            assert agg.agg_tune_table_apply(other.ctx, sh.M, sh.N, sh.K)
            assert not agg.agg_tune_table_apply(other.ctx, sh.M, sh.N, sh.K + 64)
            check_f32(other.run().cpu().numpy(), want, sh.K)
        finally:
            other.close()
    finally:
        run.close()
        agg.agg_tune_table_clear()


@pytest.mark.parametrize("K", [64, 192, 448, 960])
def test_short_and_odd_k_ranges(K):
    """One to fifteen stages of 64: fewer than the ring holds, fewer than one unrolled pass of the main loop, more."""
    sh = wl.AgGemmShape(f"ag_k{K}", 14, 2, 136, K, 232)
    inp = wl.make_ag_gemm(sh, a_dist=("int", 2), b_dist=("int", 2))
    want = oracle.ag_gemm(inp.shards, inp.B_kn, 1)
    run = AgGemmRun(inp, 1)
    try:
        for tile in range(8):
            C = run.run(tile=tile).cpu().numpy()
            assert np.array_equal(C.astype(np.float64), want), (K, tile)      # integer inputs: exact
    finally:
        run.close()


def test_b_given_as_k_by_n_is_transposed_first_same_bits():
    inp = wl.make_ag_gemm(wl.AG_RAGGED)
    sh = wl.AG_RAGGED
    run = AgGemmRun(inp, 2)
    try:
        base = run.run(tile=1).cpu().numpy()
        # the transposed copy lives in a workspace that no GEMM call allocates: without it the call is refused
        Cx = torch.zeros((sh.M, sh.N), device="cuda", dtype=torch.float32)
        with pytest.raises(agg.AggError) as e:
            agg.ag_gemm(run.ctx, sh.M, sh.N, sh.K, run.B_nk, sh.N, agg.B_KN, Cx, sh.N, agg.F32, run.cons)
        assert e.value.code == agg.ERR_NOT_RESERVED
        agg.agg_reserve_b_kn(run.ctx, sh.N, sh.K)
        for pad in (0, 3):                                   # ldb = N and ldb = N + 3 (no alignment asked of this layout)
            host = np.zeros((sh.K, sh.N + pad), dtype=np.uint16)
            host[:, : sh.N] = inp.B_kn
            B_kn = dev_bf16(host)
            run.poison()
            agg.signal_reset(run.ctx)
            C = torch.full((sh.M, sh.N), float("nan"), device="cuda", dtype=torch.float32)
            torch.cuda.synchronize()
            agg.ag_gemm(run.ctx, sh.M, sh.N, sh.K, B_kn, sh.N + pad, agg.B_KN, C, sh.N, agg.F32, run.cons)
            agg.ag_producer_emulate(run.ctx, run.remote, None, agg.PRODUCER_KERNEL, 0, run.prod)
            torch.cuda.synchronize()
            assert agg.agg_status(run.ctx) == agg.OK
            assert np.array_equal(C.cpu().numpy().view(np.uint32), base.view(np.uint32))
        with pytest.raises(agg.AggError):
            agg.ag_gemm(run.ctx, sh.M, sh.N, sh.K, B_kn, sh.N - 1, agg.B_KN, C, sh.N, agg.F32, run.cons)    # ldb < N
    finally:
        run.close()


def test_two_k_by_n_calls_on_two_streams_do_not_mix_their_operands():
    # one transposed copy per context: a second [K][N] call on another stream, with another B, must wait for the
    # first one's GEMM (the library orders them); both results are those of the [N][K] calls
    inp = wl.make_ag_gemm(wl.AG_RAGGED)
    sh = wl.AG_RAGGED
    run = AgGemmRun(inp, 1)
    try:
        agg.agg_reserve_b_kn(run.ctx, sh.N, sh.K)
        B1_kn = dev_bf16(inp.B_kn)
        neg = (inp.B_kn ^ np.uint16(0x8000)).astype(np.uint16)            # -B: same magnitudes, every sign flipped
        B2_kn = dev_bf16(neg)
        B2_nk = dev_bf16(np.ascontiguousarray(neg.T))
        run.run(tile=1)                                                    # T filled, signals of this epoch set
        ref1 = torch.empty((sh.M, sh.N), device="cuda", dtype=torch.float32)
        ref2 = torch.empty_like(ref1)
        agg.ag_gemm(run.ctx, sh.M, sh.N, sh.K, run.B_nk, sh.K, agg.B_NK, ref1, sh.N, agg.F32, run.cons)
        agg.ag_gemm(run.ctx, sh.M, sh.N, sh.K, B2_nk, sh.K, agg.B_NK, ref2, sh.N, agg.F32, run.cons)
        torch.cuda.synchronize()
        assert not torch.equal(ref1, ref2) and torch.allclose(ref2, -ref1, rtol=1e-3, atol=1e-3)
        for _ in range(3):
            C1 = torch.full((sh.M, sh.N), float("nan"), device="cuda", dtype=torch.float32)
            C2 = torch.full((sh.M, sh.N), float("nan"), device="cuda", dtype=torch.float32)
            torch.cuda.synchronize()
            agg.ag_gemm(run.ctx, sh.M, sh.N, sh.K, B1_kn, sh.N, agg.B_KN, C1, sh.N, agg.F32, run.cons)
            agg.ag_gemm(run.ctx, sh.M, sh.N, sh.K, B2_kn, sh.N, agg.B_KN, C2, sh.N, agg.F32, run.prod)
            torch.cuda.synchronize()
            assert agg.agg_status(run.ctx) == agg.OK
            assert torch.equal(C1, ref1) and torch.equal(C2, ref2)
    finally:
        run.close()


def test_seeded_random_shapes_and_settings_exact():
    """Thirty seeded combinations of world size, shard rows, K, N, signals per shard, tile shape, tile order, producer,
    own-shard handling, output type and launch order; integer inputs, so every result must equal the oracle exactly."""
    rng = np.random.default_rng(2024)
    done = 0
    while done < 30:
        W = int(rng.choice([1, 2, 3, 4, 5, 8]))
        cps = int(rng.choice([1, 2, 4]))
        Ms = max(int(rng.choice([8, 32, 64, 100, 128, 200, 256, 264, 512])) // cps * cps, cps)
        K = 64 * int(rng.integers(1, 12))
        N = int(rng.choice([8, 24, 100, 101, 128, 222, 224, 232, 256, 257, 300, 448, 520, 736]))
        rank = int(rng.integers(0, W))
        tile = int(rng.choice([-1, 0, 1, 2, 3]))
        order = int(rng.choice([agg.ORDER_ROTATED, agg.ORDER_SUBCHUNK]))
        mode = int(rng.choice([agg.PRODUCER_KERNEL, agg.PRODUCER_LINKS, agg.PRODUCER_SDMA]))
        local = bool(rng.integers(0, 2))
        out = int(rng.choice([agg.F32, agg.BF16]))
        consumer_first = bool(rng.integers(0, 2))
        if (Ms * K * 2) % (cps * 16) != 0:
            continue
        what = (W, rank, Ms, K, N, cps, tile, order, mode, local, out, consumer_first)
        print("[random case]", what, flush=True)
        sh = wl.AgGemmShape("ag_random", 50 + done, W, Ms, K, N)
        inp = wl.make_ag_gemm(sh, a_dist=("int", 2), b_dist=("int", 2))
        want = oracle.ag_gemm(inp.shards, inp.B_kn, rank)
        run = AgGemmRun(inp, rank, chunks_per_shard=cps)
        try:
            run.ctx.set_tile_order(order)
            flag = 0
            if local:
                run.ctx.set_local_shard(run.remote[rank])
                flag = agg.PRODUCER_LOCAL_LAST
            arrival = wl.arrival_orders(W, rank, limit=3, seed=done)[-1] if W > 1 else None
            C = run.run(arrival, out_dtype=out, mode=mode | flag, tile=tile, consumer_first=consumer_first)
            if out == agg.F32:
                assert np.array_equal(C.cpu().numpy().astype(np.float64), want), what
            else:
                assert np.array_equal(host_bits(C), wl.f32_to_bf16_bits(want.astype(np.float32))), what
        finally:
            run.close()
        done += 1


def test_all_ranks_on_one_gpu_assemble_the_full_product():
    """W emulated ranks, each with its own symmetric buffer, pulling the others' shards and multiplying by its own column
    slice of B: side by side the W outputs are A . B of the whole problem (Section 2.3: the tensor-parallel AG + GEMM)."""
    W, Ms, K, Nl = 4, 128, 192, 136
    rng = np.random.default_rng(77)
    A = [wl.f32_to_bf16_bits(rng.uniform(-1, 1, (Ms, K)).astype(np.float32)) for _ in range(W)]
    B = [wl.f32_to_bf16_bits(rng.normal(0, 0.05, (K, Nl)).astype(np.float32)) for _ in range(W)]
    want = oracle.gemm(np.concatenate(A), np.concatenate(B, axis=1))
    from harness import dev_bf16
    L = [dev_bf16(a) for a in A]                                   # rank r's local shard: every rank pulls from these
    Bd = [dev_bf16(np.ascontiguousarray(b.T)) for b in B]
    ctxs = [agg.symm_alloc(W, r, Ms * K * 2, 2 * W) for r in range(W)]
    C = [torch.full((W * Ms, Nl), float("nan"), device="cuda", dtype=torch.float32) for _ in range(W)]
    try:
        for r, ctx in enumerate(ctxs):
            agg.signal_reset(ctx)
            ps, cs = ctx.streams()
            # producers first: eight streams share the device's few hardware queues
            agg.ag_producer_emulate(ctx, L, None, agg.PRODUCER_KERNEL if r % 2 else agg.PRODUCER_LINKS, 0, ps)
        for r, ctx in enumerate(ctxs):
            ps, cs = ctx.streams()
            agg.ag_gemm(ctx, W * Ms, Nl, K, Bd[r], K, agg.B_NK, C[r], Nl, agg.F32, cs)
        torch.cuda.synchronize()
        for ctx in ctxs:
            assert agg.agg_status(ctx) == agg.OK
        got = torch.cat(C, dim=1).cpu().numpy()
        check_f32(got, want, K)
    finally:
        for ctx in ctxs:
            ctx.free()

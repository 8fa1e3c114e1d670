"""GPU parity of the MoE AllGather grouped GEMM (Section 4.1, Table 4) against the CPU oracle, through the C ABI.

Routing outputs (sorted tokens, segment offsets) are integer work: bit-exact.  Y on the fp32 path: rel. Frobenius
<= 1e-4 and max abs <= 1e-3*sqrt(K) against the fp64 oracle; the bf16 path equals RNE of the fp32 path bit for bit.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2504_19442_amd as agg
import workloads as wl
from harness import dev_bf16, host_bits, _tensor_from_ptr

pytestmark = pytest.mark.gpu


class MoeRun:
    def __init__(self, inp, rank, chunks_per_shard=1):
        sh = inp.shape
        self.inp, self.sh, self.rank = inp, sh, rank
        self.remote = [dev_bf16(s) for s in inp.shards]
        # weights as [E][N][K] (K contiguous), the layout the boundary takes
        self.Wd = dev_bf16(np.ascontiguousarray(np.transpose(inp.W_ekn, (0, 2, 1))))
        self.ids = torch.from_numpy(inp.topk_ids).cuda()
        self.ctx = agg.symm_alloc(sh.W, rank, sh.tokens_per_rank * sh.K * 2, sh.W * chunks_per_shard)
        agg.agg_reserve_moe(self.ctx, sh.T, sh.topk, sh.E, sh.N)
        ps, cs = self.ctx.streams()
        self.prod, self.cons = torch.cuda.ExternalStream(ps), torch.cuda.ExternalStream(cs)
        self.staging = _tensor_from_ptr(self.ctx.staging, sh.T * sh.K)

    def run(self, order=None, out_dtype=agg.F32, tile=None, consumer_first=True, ldy=None):
        sh = self.sh
        P = sh.T * sh.topk
        ldy = ldy or sh.N
        self.staging.fill_(float("nan"))
        if tile is not None:
            self.ctx.set_tile_config(tile)
        agg.signal_reset(self.ctx)
        Y = torch.full((P, ldy), float("nan"), device="cuda",
                       dtype=torch.float32 if out_dtype == agg.F32 else torch.bfloat16)
        tok = torch.full((P,), -7, device="cuda", dtype=torch.int32)
        seg = torch.full((sh.E + 1,), -7, device="cuda", dtype=torch.int32)
        torch.cuda.synchronize()

        def consume():
            agg.ag_moe_gemm(self.ctx, sh.T, sh.topk, sh.E, sh.N, sh.K, self.ids, self.Wd, tok, seg, Y, ldy,
                            out_dtype, self.cons)

        def produce():
            agg.ag_producer_emulate(self.ctx, self.remote, order, agg.PRODUCER_KERNEL, 0, self.prod)

        if consumer_first:
            consume(); produce()
        else:
            produce(); consume()
        torch.cuda.synchronize()
        st = agg.agg_status(self.ctx)
        assert st == agg.OK, agg.agg_strerror(st)
        return Y, tok.cpu().numpy(), seg.cpu().numpy()

    def close(self):
        self.ctx.free()


def _check_y(Y, want, K):
    got = Y.astype(np.float64)
    rel = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30)
    assert rel <= 1e-4, rel
    assert np.abs(got - want).max() <= 1e-3 * np.sqrt(K)


@pytest.mark.parametrize("rank", [0, 2])
@pytest.mark.parametrize("tile", list(range(8)))
def test_moe_tiny_against_oracle(rank, tile):
    sh = wl.MOE_TINY
    inp = wl.make_moe(sh)
    tok_ref, slot_ref, seg_ref = oracle.moe_route(inp.topk_ids, sh.E)
    want = oracle.moe_gemm(inp.shards, inp.W_ekn, inp.topk_ids, rank)
    run = MoeRun(inp, rank)
    try:
        base = None
        orders = wl.arrival_orders(sh.W, rank, limit=4, seed=3)
        for k, order in enumerate(orders):
            Y, tok, seg = run.run(order=list(order), tile=tile, consumer_first=(k % 2 == 0))
            assert np.array_equal(tok, tok_ref)
            assert np.array_equal(seg.astype(np.int64), seg_ref)
            y = Y.cpu().numpy()
            assert not np.isnan(y).any()
            _check_y(y, want, sh.K)
            if base is None:
                base = y
            else:
                assert np.array_equal(base.view(np.uint32), y.view(np.uint32))   # arrival order changes nothing
        Yb, _, _ = run.run(out_dtype=agg.BF16, tile=tile)
        assert np.array_equal(host_bits(Yb), wl.f32_to_bf16_bits(base))
        # padded leading dimension: the padding columns stay untouched
        Yp, _, _ = run.run(tile=tile, ldy=sh.N + 8)
        yp = Yp.cpu().numpy()
        assert np.array_equal(yp[:, :sh.N].view(np.uint32), base.view(np.uint32))
        assert np.isnan(yp[:, sh.N:]).all()
    finally:
        run.close()


def test_moe_integer_inputs_exact_and_several_signals_per_shard():
    sh = wl.MOE_TINY
    inp = wl.make_moe(sh, x_dist=("int", 2), w_dist=("int", 2))
    want = oracle.moe_gemm(inp.shards, inp.W_ekn, inp.topk_ids, 1)
    run = MoeRun(inp, 1, chunks_per_shard=4)
    try:
        Y, _, _ = run.run()
        assert np.array_equal(Y.cpu().numpy().astype(np.float64), want)
    finally:
        run.close()


@pytest.mark.parametrize("tile", [0, 2, 3])
def test_moe_segments_with_full_blocks_and_short_tails(tile):
    # 640 tokens x top-2 over 5 experts, 150 pairs moved from expert 4 to expert 3.  Rows per expert: 276 and 261 (a full
    # 256-row block and a short tail for the 128-row launch), 242 (one 256-row tile), 399 (a full block and a tail of
    # 143 rows), 102 (less than half a tile).  Integer inputs: the result is exact.
    sh = wl.MoeShape("moe_blocks", 17, 2, 320, 128, 320, 5, 2)
    inp = wl.make_moe(sh, x_dist=("int", 2), w_dist=("int", 2))
    ids = inp.topk_ids.copy()
    for col in (0, 1):
        move = np.nonzero((ids[:, col] == 4) & (ids[:, 1 - col] != 3))[0][:75]
        ids[move, col] = 3
    inp = wl.MoeInputs(sh, inp.shards, inp.W_ekn, np.ascontiguousarray(ids))
    counts = np.bincount(ids.reshape(-1), minlength=sh.E)
    assert list(counts) == [276, 242, 261, 399, 102], counts
    want = oracle.moe_gemm(inp.shards, inp.W_ekn, inp.topk_ids, 1)
    run = MoeRun(inp, 1, chunks_per_shard=2)
    try:
        Y, tok, seg = run.run(tile=tile)
        assert np.array_equal(np.diff(seg), counts)
        assert np.array_equal(Y.cpu().numpy().astype(np.float64), want)
    finally:
        run.close()


@pytest.mark.parametrize("W,tpr,E,topk", [(2, 4600, 2, 2), (3, 5463, 3, 1)])
def test_moe_long_segments_and_more_pairs_than_one_pass_of_the_routing_holds(W, tpr, E, topk):
    # 18400 pairs (a multiple of four) and 16389 (not one): more than the 16384 ids the routing kernel takes at a time,
    # and segments of more than 4096 rows (longer than what it keeps on chip for the tile table).  Integer inputs: exact.
    sh = wl.MoeShape("moe_long", 21, W, tpr, 64, 64, E, topk)
    inp = wl.make_moe(sh, x_dist=("int", 2), w_dist=("int", 2))
    want = oracle.moe_gemm(inp.shards, inp.W_ekn, inp.topk_ids, 0)
    tok_ref, _, seg_ref = oracle.moe_route(inp.topk_ids, sh.E)
    assert np.diff(seg_ref).max() > 4096 and sh.T * sh.topk > 16384
    run = MoeRun(inp, 0)
    try:
        Y, tok, seg = run.run()
        assert np.array_equal(tok, tok_ref)
        assert np.array_equal(seg.astype(np.int64), seg_ref)
        assert np.array_equal(Y.cpu().numpy().astype(np.float64), want)
    finally:
        run.close()


def test_moe_more_experts_than_routing_workgroups_fit_on_the_chip_at_once():
    # 1000 experts = 1000 routing workgroups of 16 waves: more than are resident together, so late workgroups read the
    # counts of workgroups that have long finished.  Most experts get a handful of rows, some none.  Three runs: the
    # routing's counters go back to rest after every call.
    sh = wl.MoeShape("moe_many_experts", 23, 1, 5000, 64, 8, 1000, 1)
    inp = wl.make_moe(sh, x_dist=("int", 2), w_dist=("int", 2))
    want = oracle.moe_gemm(inp.shards, inp.W_ekn, inp.topk_ids, 0)
    tok_ref, _, seg_ref = oracle.moe_route(inp.topk_ids, sh.E)
    run = MoeRun(inp, 0)
    try:
        for _ in range(3):
            Y, tok, seg = run.run()
            assert np.array_equal(tok, tok_ref)
            assert np.array_equal(seg.astype(np.int64), seg_ref)
            assert np.array_equal(Y.cpu().numpy().astype(np.float64), want)
    finally:
        run.close()


def test_moe_empty_experts_skewed_routing_and_invalid_ids():
    sh = wl.MoeShape("moe_skew", 9, 2, 40, 64, 40, 7, 2)
    inp = wl.make_moe(sh)
    ids = inp.topk_ids.copy()
    # experts 3 and 6 get nothing; expert 0 gets every token; one pair carries an invalid id and is skipped
    ids[:, 0] = 0
    ids[:, 1] = np.where(np.isin(ids[:, 1], (0, 3, 6)), 1, ids[:, 1])
    ids[5, 1] = 99
    inp = wl.MoeInputs(sh, inp.shards, inp.W_ekn, np.ascontiguousarray(ids))
    valid = ids.copy()
    run = MoeRun(inp, 0)
    try:
        Y, tok, seg = run.run()
        P = sh.T * sh.topk
        # reference routing written out directly: stable order of the flat pair index per expert
        flat = valid.reshape(-1)
        ref_tok, ref_seg = [], [0]
        for e in range(sh.E):
            idx = np.nonzero(flat == e)[0]
            ref_tok += list(idx // sh.topk)
            ref_seg.append(ref_seg[-1] + len(idx))
        assert list(seg) == ref_seg and seg[-1] == P - 1
        assert list(tok[:P - 1]) == ref_tok
        assert seg[3] == seg[4] and seg[6] == seg[7]
        # every written row against the oracle's GEMM of its (token, expert); the row past the end is untouched
        y = Y.cpu().numpy()
        X = np.concatenate([wl.bf16_bits_to_f32(s).astype(np.float64) for s in inp.shards])
        for e in range(sh.E):
            rows = np.arange(ref_seg[e], ref_seg[e + 1])
            if len(rows) == 0:
                continue
            want = oracle.gemm(wl.f32_to_bf16_bits(X[np.asarray(ref_tok)[rows]].astype(np.float32)), inp.W_ekn[e])
            _check_y(y[rows], want, sh.K)
        assert np.isnan(y[P - 1]).all()
    finally:
        run.close()


def test_moe_argument_errors():
    sh = wl.MOE_TINY
    inp = wl.make_moe(sh)
    run = MoeRun(inp, 0)
    try:
        P = sh.T * sh.topk
        Y = torch.zeros((P, sh.N), device="cuda", dtype=torch.float32)
        tok = torch.zeros((P,), device="cuda", dtype=torch.int32)
        seg = torch.zeros((sh.E + 1,), device="cuda", dtype=torch.int32)
        good = dict(Ttok=sh.T, topk=sh.topk, E=sh.E, N=sh.N, K=sh.K)
        def call(**kw):
            a = dict(good); a.update(kw)
            agg.ag_moe_gemm(run.ctx, a["Ttok"], a["topk"], a["E"], a["N"], a["K"], run.ids, run.Wd, tok, seg, Y,
                            a.get("ldy", sh.N), a.get("dt", agg.F32), run.cons)
        for bad in (dict(K=sh.K + 32), dict(Ttok=sh.T + 1), dict(topk=0), dict(E=0), dict(ldy=sh.N - 1), dict(dt=5),
                    dict(K=sh.K * 2)):
            with pytest.raises(agg.AggError):
                call(**bad)
        call(N=0)            # empty: a no-op
    finally:
        run.close()


def test_moe_full_size_whole_output():
    sh = wl.MOE_FULL
    inp = wl.make_moe(sh)
    rank = 3
    tok_ref, slot_ref, seg_ref = oracle.moe_route(inp.topk_ids, sh.E)
    run = MoeRun(inp, rank, chunks_per_shard=4)
    try:
        Y, tok, seg = run.run(out_dtype=agg.F32)
        assert np.array_equal(tok, tok_ref)
        assert np.array_equal(seg.astype(np.int64), seg_ref)
        # every row of Y (all experts, all tiles) against the oracle
        want = oracle.moe_gemm(inp.shards, inp.W_ekn, inp.topk_ids, rank)
        _check_y(Y.cpu().numpy(), want, sh.K)
        Y2, _, _ = run.run(out_dtype=agg.F32, order=list(wl.arrival_orders(sh.W, rank, limit=2, seed=4)[-1]),
                           consumer_first=False)
        assert torch.equal(Y, Y2)
    finally:
        run.close()


def test_moe_call_without_a_reserved_workspace_is_refused():
    sh = wl.MOE_TINY
    inp = wl.make_moe(sh)
    run = MoeRun(inp, 0)
    bare = agg.symm_alloc(sh.W, 0, sh.tokens_per_rank * sh.K * 2, sh.W)       # a context nobody reserved anything for
    try:
        P = sh.T * sh.topk
        Y = torch.zeros((P, sh.N), device="cuda", dtype=torch.float32)
        tok = torch.zeros((P,), device="cuda", dtype=torch.int32)
        seg = torch.zeros((sh.E + 1,), device="cuda", dtype=torch.int32)
        ids = torch.from_numpy(inp.topk_ids).cuda()
        with pytest.raises(agg.AggError) as e:
            agg.ag_moe_gemm(bare, sh.T, sh.topk, sh.E, sh.N, sh.K, ids, run.Wd, tok, seg, Y, sh.N, agg.F32, None)
        assert e.value.code == agg.ERR_NOT_RESERVED
        # a reserved context: the very first call (no warm call before it) goes through
        run.run(out_dtype=agg.F32)
        # a workspace reserved for a smaller problem is refused as well
        agg.agg_reserve_moe(bare, sh.W, 1, 1, 16)
        with pytest.raises(agg.AggError) as e:
            agg.ag_moe_gemm(bare, sh.T, sh.topk, sh.E, sh.N, sh.K, ids, run.Wd, tok, seg, Y, sh.N, agg.F32, None)
        assert e.value.code == agg.ERR_NOT_RESERVED
    finally:
        bare.free()
        run.close()

"""ag_moe_gemm_static (the entry point that allocates nothing: its tile table lives in a fixed device array of the
library) against ag_moe_gemm on the same inputs, through the C ABI: two calls in a row, the second on a smaller problem."""
import numpy as np
import pytest
import torch

import paper_2504_19442_amd as agg
import workloads as wl
from harness import dev_bf16

pytestmark = pytest.mark.gpu


def _one(shape, rank, entry, reserve):
    """Routing + gated grouped GEMM of `shape` through `entry`; returns (Y, sorted_token, segment offsets) on the host."""
    inp = wl.make_moe(shape)
    remote = [dev_bf16(x) for x in inp.shards]
    Wd = dev_bf16(np.ascontiguousarray(np.transpose(inp.W_ekn, (0, 2, 1))))
    ids = torch.from_numpy(inp.topk_ids).cuda()
    P = shape.T * shape.topk
    Y = torch.full((P, shape.N), float("nan"), device="cuda", dtype=torch.float32)
    tok = torch.full((P,), -7, device="cuda", dtype=torch.int32)
    seg = torch.full((shape.E + 1,), -7, device="cuda", dtype=torch.int32)
    ctx = agg.symm_alloc(shape.W, rank, shape.tokens_per_rank * shape.K * 2, shape.W)
    try:
        if reserve:
            agg.agg_reserve_moe(ctx, shape.T, shape.topk, shape.E, shape.N)
        ps, cs = ctx.streams()
        agg.signal_reset(ctx)
        torch.cuda.synchronize()
        entry(ctx, shape.T, shape.topk, shape.E, shape.N, shape.K, ids, Wd, tok, seg, Y, shape.N, agg.F32, cs)
        agg.ag_producer_emulate(ctx, remote, None, agg.PRODUCER_KERNEL, 0, ps)
        torch.cuda.synchronize()
        assert agg.agg_status(ctx) == agg.OK
    finally:
        ctx.free()
    return Y.cpu().numpy(), tok.cpu().numpy(), seg.cpu().numpy()


def test_static_scratch_entry_point_matches_the_allocating_one_twice_in_a_row():
    big = wl.MoeShape("moe_static_a", 31, 4, 96, 256, 384, 12, 2)      # 384 tokens, 12 experts: ragged segments
    small = wl.MoeShape("moe_static_b", 32, 2, 40, 128, 136, 3, 2)     # then a smaller problem: fewer tiles, other shapes
    for shape, rank in ((big, 1), (small, 0)):
        want = _one(shape, rank, agg.ag_moe_gemm, reserve=True)
        got = _one(shape, rank, agg.ag_moe_gemm_static, reserve=False)  # nothing reserved: the static array is all it has
        assert np.array_equal(got[1], want[1]) and np.array_equal(got[2], want[2])
        assert not np.isnan(got[0][: want[2][-1]]).any()
        assert np.array_equal(got[0].view(np.uint32), want[0].view(np.uint32))


def test_static_scratch_entry_point_refuses_a_table_beyond_its_array():
    shape = wl.MOE_TINY
    ctx = agg.symm_alloc(shape.W, 0, shape.tokens_per_rank * shape.K * 2, shape.W)
    try:
        z = torch.zeros(64, device="cuda", dtype=torch.int32)
        with pytest.raises(agg.AggError) as e:      # 2^20 tokens x 64 columns of 128: far more than 32760 table entries
            agg.ag_moe_gemm_static(ctx, shape.W << 18, 2, 64, 8192, shape.K, z, z, z, z, z, 8192, agg.F32, None)
        assert e.value.code == agg.ERR_UNSUPPORTED_SHAPE
    finally:
        ctx.free()

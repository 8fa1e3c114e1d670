"""GPU parity of MoE + ReduceScatter (grouped GEMM, top-k reduction, reduce scatter) against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2504_19442_amd as agg
import workloads as wl
from harness import dev_bf16

pytestmark = pytest.mark.gpu


class MoeRsRun:
    def __init__(self, inp, rank, chunks=1):
        sh = inp.shape
        self.inp, self.sh, self.rank = inp, sh, rank
        self.H = dev_bf16(inp.H)
        self.W2 = dev_bf16(np.ascontiguousarray(np.transpose(inp.W2_ekn, (0, 2, 1))))      # [E][N][Kl]
        self.ids = torch.from_numpy(inp.topk_ids).cuda()
        self.gate = torch.from_numpy(inp.gate).cuda()
        self.chunks = chunks
        self.ctx = agg.symm_alloc(sh.W, rank, 16, sh.W * chunks)
        agg.agg_reserve_moe(self.ctx, sh.T, sh.topk, sh.E, sh.N)
        self.ctx.set_rs_chunks(chunks)
        ps, cs = self.ctx.streams()
        self.prod, self.cons = torch.cuda.ExternalStream(ps), torch.cuda.ExternalStream(cs)
        P = sh.T * sh.topk
        self.Y = torch.empty((P, sh.N), device="cuda", dtype=torch.float32)
        self.tok = torch.empty((P,), device="cuda", dtype=torch.int32)
        self.seg = torch.empty((sh.E + 1,), device="cuda", dtype=torch.int32)
        self.pos = torch.empty((P,), device="cuda", dtype=torch.int32)
        self.slots = [torch.full((sh.tokens_per_rank, sh.N), float("nan"), device="cuda", dtype=torch.float32)
                      for _ in range(sh.W)]
        self.peers = {w: torch.from_numpy(s).cuda() for w, s in inp.peer_slots.items()}

    def run(self, peers_first, with_other=True, r_dtype=agg.F32, tile=None):
        sh = self.sh
        for s in self.slots:
            s.fill_(float("nan"))
        self.Y.fill_(float("nan"))
        if tile is not None:
            self.ctx.set_tile_config(tile)
        agg.signal_reset(self.ctx)
        Z = torch.full((sh.T, sh.N), float("nan"), device="cuda", dtype=torch.float32) if with_other else None
        R = torch.full((sh.tokens_per_rank, sh.N), float("nan"), device="cuda",
                       dtype=torch.float32 if r_dtype == agg.F32 else torch.bfloat16)
        torch.cuda.synchronize()

        def deliver():
            for w in sorted(self.peers, reverse=True):
                with torch.cuda.stream(self.prod):
                    self.slots[w].copy_(self.peers[w], non_blocking=True)
                for c in range(self.chunks):
                    agg.signal_set(self.ctx, w * self.chunks + c, self.prod)

        if peers_first:
            deliver()
        agg.moe_rs(self.ctx, sh.T, sh.topk, sh.E, sh.N, sh.Kl, self.H, self.W2, self.ids, self.gate, self.Y, self.tok,
                   self.seg, self.pos, self.slots, Z, R, sh.N, r_dtype, self.prod, self.cons)
        if not peers_first:
            deliver()
        torch.cuda.synchronize()
        st = agg.agg_status(self.ctx)
        assert st == agg.OK, agg.agg_strerror(st)
        return R, Z

    def close(self):
        self.ctx.free()


def _close(got, want, K):
    rel = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30)
    assert rel <= 1e-4, rel
    assert np.abs(got - want).max() <= 1e-3 * np.sqrt(K)


@pytest.mark.parametrize("rank", [0, 2])
@pytest.mark.parametrize("tile", list(range(8)))
def test_moe_rs_tiny(rank, tile):
    sh = wl.MOE_RS_TINY
    inp = wl.make_moe_rs(sh, rank=rank)
    want = oracle.moe_rs(inp.H, inp.W2_ekn, inp.topk_ids, inp.gate, inp.peer_slots, sh.W, rank)
    tok_ref, slot_ref, seg_ref = oracle.moe_route(inp.topk_ids, sh.E)
    run = MoeRsRun(inp, rank)
    try:
        base = None
        for peers_first in (False, True):
            R, Z = run.run(peers_first, tile=tile)
            r = R.cpu().numpy()
            _close(r.astype(np.float64), want, sh.Kl)
            if base is None:
                base = r
            else:
                assert np.array_equal(base.view(np.uint32), r.view(np.uint32))       # arrival changes nothing
        # routing outputs, bit for bit
        assert np.array_equal(run.tok.cpu().numpy(), tok_ref)
        assert np.array_equal(run.seg.cpu().numpy().astype(np.int64), seg_ref)
        pos = run.pos.cpu().numpy().reshape(sh.T, sh.topk)
        for p in range(sh.T * sh.topk):
            assert pos[tok_ref[p], slot_ref[p]] == p
        # the result is the ordered fp32 sum of the slots as they stand on the device
        slots = [s.cpu().numpy() for s in run.slots]
        assert np.array_equal(oracle.rs_reduce_f32(slots).view(np.uint32), base.view(np.uint32))
        # the other ranks' tokens: top-k reduction alone (no peers), against the oracle with zero peer slices
        z = Z.cpu().numpy()
        Tr = sh.tokens_per_rank
        assert np.isnan(z[rank * Tr:(rank + 1) * Tr]).all()                          # own rows went to the slot
        zero = {w: np.zeros((Tr, sh.N), dtype=np.float32) for w in range(sh.W)}
        for other in range(sh.W):
            if other == rank:
                continue
            zw = {w: s for w, s in zero.items() if w != other}
            ref = oracle.moe_rs(inp.H, inp.W2_ekn, inp.topk_ids, inp.gate, zw, sh.W, other)
            _close(z[other * Tr:(other + 1) * Tr].astype(np.float64), ref, sh.Kl)
        # bf16 result = RNE of the fp32 result; Z_other may be left out
        Rb, _ = run.run(True, with_other=False, r_dtype=agg.BF16, tile=tile)
        from harness import host_bits
        assert np.array_equal(host_bits(Rb), wl.f32_to_bf16_bits(base))
    finally:
        run.close()


def test_moe_rs_three_experts_per_token():
    # three pairs per token: the reduction adds the three products in slot order (the same bits in every run)
    sh = wl.MoeRsShape("moe_rs_top3", 19, 2, 48, 128, 72, 6, 3)
    inp = wl.make_moe_rs(sh, rank=1)
    want = oracle.moe_rs(inp.H, inp.W2_ekn, inp.topk_ids, inp.gate, inp.peer_slots, sh.W, 1)
    run = MoeRsRun(inp, 1)
    try:
        R1, _ = run.run(False)
        _close(R1.cpu().numpy().astype(np.float64), want, sh.Kl)
        R2, _ = run.run(True)
        assert torch.equal(R1, R2)
    finally:
        run.close()


def test_moe_rs_long_segments_exact():
    # every token goes to both experts: segments of 9200 rows, 18400 pairs; without Z_other only the rows of this
    # rank's tokens are computed (one run of rows in the middle of each segment)
    sh = wl.MoeRsShape("moe_rs_long", 22, 2, 4600, 64, 64, 2, 2)
    inp = wl.make_moe_rs(sh, rank=1, h_dist=("int", 2), w_dist=("int", 2), slot_dist=("int", 3))
    inp.gate[:] = np.float32(0.5)
    want = oracle.moe_rs(inp.H, inp.W2_ekn, inp.topk_ids, inp.gate, inp.peer_slots, sh.W, 1)
    run = MoeRsRun(inp, 1)
    try:
        for with_other in (False, True):
            R, _ = run.run(True, with_other=with_other)
            assert np.array_equal(R.cpu().numpy().astype(np.float64), want)
    finally:
        run.close()


@pytest.mark.parametrize("chunks", [1, 4])
def test_moe_rs_integer_inputs_exact(chunks):
    sh = wl.MoeRsShape("moe_rs_int", 18, 2, 40, 128, 40, 7, 2)
    inp = wl.make_moe_rs(sh, rank=1, h_dist=("int", 2), w_dist=("int", 2), slot_dist=("int", 3))
    inp.gate[:] = np.float32(0.5)                     # halves: every product and sum below is exact in fp32
    want = oracle.moe_rs(inp.H, inp.W2_ekn, inp.topk_ids, inp.gate, inp.peer_slots, sh.W, 1)
    run = MoeRsRun(inp, 1, chunks=chunks)       # with chunks: every slot is signalled in four row chunks of 10 tokens
    try:
        R, _ = run.run(False)
        assert np.array_equal(R.cpu().numpy().astype(np.float64), want)
        if chunks > 1:
            run.ctx.set_rs_chunks(3)             # 40 tokens per rank do not cut into 3 chunks: refused before any launch
            with pytest.raises(agg.AggError):
                run.run(False)
    finally:
        run.close()


def test_moe_rs_argument_errors():
    sh = wl.MOE_RS_TINY
    inp = wl.make_moe_rs(sh, rank=0)
    run = MoeRsRun(inp, 0)
    try:
        R = torch.zeros((sh.tokens_per_rank, sh.N), device="cuda", dtype=torch.float32)
        def call(**kw):
            a = dict(T=sh.T, topk=sh.topk, E=sh.E, N=sh.N, K=sh.Kl, slots=run.slots, ldr=sh.N, dt=agg.F32)
            a.update(kw)
            agg.moe_rs(run.ctx, a["T"], a["topk"], a["E"], a["N"], a["K"], run.H, run.W2, run.ids, run.gate, run.Y, run.tok,
                       run.seg, run.pos, a["slots"], None, R, a["ldr"], a["dt"], run.prod, run.cons)
        for bad in (dict(K=sh.Kl + 32), dict(T=sh.T + 1), dict(topk=0), dict(E=0), dict(N=sh.N + 2), dict(ldr=sh.N - 4),
                    dict(dt=9), dict(slots=run.slots[:3] + [None])):
            with pytest.raises(agg.AggError):
                call(**bad)
        call(N=0)
    finally:
        run.close()


def test_moe_rs_full_size_all_tokens_of_the_rank():
    sh = wl.MOE_RS_FULL
    rank = 6
    inp = wl.make_moe_rs(sh, rank=rank)
    rows = np.arange(sh.tokens_per_rank)          # the whole of R
    want = oracle.moe_rs(inp.H, inp.W2_ekn, inp.topk_ids, inp.gate, inp.peer_slots, sh.W, rank, rows=rows)
    run = MoeRsRun(inp, rank)
    try:
        R, Z = run.run(False)
        r = R.cpu().numpy()
        assert not np.isnan(r).any()
        _close(r[rows].astype(np.float64), want, sh.Kl)
        R2, _ = run.run(True, with_other=False)
        assert torch.equal(R, R2)
    finally:
        run.close()


def test_moe_rs_pair_with_an_invalid_expert_id_contributes_nothing():
    sh = wl.MOE_RS_TINY
    inp = wl.make_moe_rs(sh, rank=0)
    t_bad, s_bad = 7, 1
    # the oracle's view: the same routing, but that pair's gate is zero
    gate0 = inp.gate.copy(); gate0[t_bad, s_bad] = 0.0
    want = oracle.moe_rs(inp.H, inp.W2_ekn, inp.topk_ids, gate0, inp.peer_slots, sh.W, 0)
    # the GPU's view: the id itself is invalid, so the pair drops out of the sorted order; H keeps one row per valid
    # pair in that (shorter) order
    tok, slot, seg = oracle.moe_route(inp.topk_ids, sh.E)
    keep = [p for p in range(sh.T * sh.topk) if not (tok[p] == t_bad and slot[p] == s_bad)]
    H2 = np.zeros_like(inp.H); H2[: len(keep)] = inp.H[keep]
    ids2 = inp.topk_ids.copy(); ids2[t_bad, s_bad] = 1000
    bad = wl.MoeRsInputs(sh, H2, inp.W2_ekn, ids2, inp.gate, inp.peer_slots)
    run = MoeRsRun(bad, 0)
    try:
        R, _ = run.run(True, with_other=False)
        _close(R.cpu().numpy().astype(np.float64), want, sh.Kl)
        assert run.pos.cpu().numpy().reshape(sh.T, sh.topk)[t_bad, s_bad] == -1
        assert run.seg.cpu().numpy()[-1] == sh.T * sh.topk - 1
    finally:
        run.close()

"""Pins for the oracle's ReduceScatter reduction, GEMM+RS and MoE grouped GEMM (no GPU)."""
import math
import os

import numpy as np
import pytest

import oracle
import workloads as wl
from test_oracle_gemm import _read_golden, bits, widen


# ---------------------------------------------------------------- reducer


def test_rs_order_fixture():
    g = _read_golden("rs_order_f32.txt")
    slots = [np.array([v], dtype=np.float32) for v in g["slots"]]
    assert oracle.rs_reduce_f32(slots)[0] == g["f32_in_order"][0]
    assert oracle.rs_reduce_f64(slots)[0] == g["f64_exact"][0]
    assert oracle.rs_reduce_f32(slots[::-1])[0] == g["f32_reversed"][0]


def test_rs_f64_is_exact_sum():
    rng = np.random.default_rng(21)
    W, n = 8, 257
    slots = [rng.standard_normal(n).astype(np.float32) for _ in range(W)]
    got = oracle.rs_reduce_f64(slots)
    for i in range(n):
        exact = math.fsum(float(s[i]) for s in slots)
        assert abs(got[i] - exact) <= 8 * 2.0**-53 * sum(abs(float(s[i])) for s in slots)


def test_rs_f32_matches_sequential_numpy_float32():
    rng = np.random.default_rng(22)
    W, shape = 8, (33, 65)
    slots = [rng.standard_normal(shape).astype(np.float32) for _ in range(W)]
    acc = np.zeros(shape, dtype=np.float32)
    for s in slots:                      # numpy float32 addition is IEEE, one rounding per add
        acc = acc + s
    got = oracle.rs_reduce_f32(slots)
    assert got.dtype == np.float32 and np.array_equal(got, acc)
    # and it sits within the fp32 forward-error bound of the exact sum
    exact = oracle.rs_reduce_f64(slots)
    bound = (W - 1) * 2.0**-24 * np.sum([np.abs(s).astype(np.float64) for s in slots], axis=0) * 1.01
    assert np.all(np.abs(got.astype(np.float64) - exact) <= bound)


def test_rs_w1_is_copy_and_integers_are_exact():
    rng = np.random.default_rng(23)
    s = rng.standard_normal((5, 7)).astype(np.float32)
    assert np.array_equal(oracle.rs_reduce_f32([s]), s)
    ints = [rng.integers(-1000, 1000, (16, 16)).astype(np.float32) for _ in range(6)]
    want = np.sum([i.astype(np.int64) for i in ints], axis=0)
    assert np.array_equal(oracle.rs_reduce_f32(ints).astype(np.int64), want)
    assert np.array_equal(oracle.rs_reduce_f64(ints).astype(np.int64), want)


def test_rs_required_bandwidth_matches_paper():
    g = _read_golden("rs_reducer_bandwidth.txt")
    v = oracle.rs_required_bandwidth(int(g["W"][0]), g["link_GBps"][0], g["nic_GBps"][0])
    assert v > g["paper_lower_bound_GBps"][0]
    assert abs(v - g["hand_value_GBps"][0]) < 0.01


# ---------------------------------------------------------------- GEMM+RS


def test_gemm_rs_equals_gemm_over_concatenated_k():
    # If every peer's slot is itself the partial product over that peer's K-chunk, the
    # ReduceScatter output is the GEMM over the whole K (integer inputs: all sums exact).
    rng = np.random.default_rng(31)
    W, M, Kl, N = 4, 32, 24, 20
    Ms = M // W
    A = rng.integers(-2, 3, (M, W * Kl)).astype(np.float32)
    B = rng.integers(-2, 3, (W * Kl, N)).astype(np.float32)
    whole = A.astype(np.int64) @ B.astype(np.int64)
    for rank in range(W):
        slots = {}
        for w in range(W):
            if w != rank:
                part = A[:, w * Kl:(w + 1) * Kl].astype(np.int64) @ B[w * Kl:(w + 1) * Kl].astype(np.int64)
                slots[w] = part[rank * Ms:(rank + 1) * Ms].astype(np.float32)
        got = oracle.gemm_rs(bits(A[:, rank * Kl:(rank + 1) * Kl]), bits(B[rank * Kl:(rank + 1) * Kl]),
                             slots, W, rank)
        assert np.array_equal(got, whole[rank * Ms:(rank + 1) * Ms].astype(np.float64))


def test_gemm_rs_decomposes_into_gemm_plus_reduction():
    inp = wl.make_gemm_rs(wl.RS_TINY, rank=1)
    sh = inp.shape
    got = oracle.gemm_rs(inp.A_loc, inp.B_kn, inp.peer_slots, sh.W, 1)
    part = (widen(inp.A_loc) @ widen(inp.B_kn))[sh.Ms:2 * sh.Ms]      # numpy fp64 matmul
    want = part + np.sum([inp.peer_slots[w].astype(np.float64) for w in inp.peer_slots], axis=0)
    assert np.max(np.abs(got - want)) <= 1e-12
    rows = np.array([3, 0, sh.Ms - 1])
    assert np.array_equal(oracle.gemm_rs(inp.A_loc, inp.B_kn, inp.peer_slots, sh.W, 1, rows=rows), got[rows])


# -------------------------------------------------------------------- MoE


def test_moe_route_is_sorted_by_expert_token_slot():
    inp = wl.make_moe(wl.MOE_TINY)
    sh = inp.shape
    ids = inp.topk_ids
    assert all(len(set(r)) == sh.topk for r in ids.tolist())          # distinct experts per token
    tok, slot, seg = oracle.moe_route(ids, sh.E)
    pairs = sorted((int(ids[t, s]), t, s) for t in range(sh.T) for s in range(sh.topk))
    assert [(int(ids[t, s]), int(t), int(s)) for t, s in zip(tok, slot)] == pairs
    counts = np.bincount(ids.ravel(), minlength=sh.E)
    assert np.array_equal(np.diff(seg), counts) and seg[0] == 0 and seg[-1] == sh.T * sh.topk


def test_moe_segments_equal_plain_gemms():
    inp = wl.make_moe(wl.MOE_TINY)
    sh = inp.shape
    X = np.concatenate([widen(s) for s in inp.shards])
    Y = oracle.moe_gemm(inp.shards, inp.W_ekn, inp.topk_ids, rank=1)
    tok, slot, seg = oracle.moe_route(inp.topk_ids, sh.E)
    assert Y.shape == (sh.T * sh.topk, sh.N)
    for e in range(sh.E):
        rows = tok[seg[e]:seg[e + 1]]
        want = X[rows] @ widen(inp.W_ekn[e])
        assert np.max(np.abs(Y[seg[e]:seg[e + 1]] - want), initial=0.0) <= 1e-12
    # un-sorting gives the per-token loop's rows
    for p in (0, 17, sh.T * sh.topk - 1):
        t, s = int(tok[p]), int(slot[p])
        want = X[t] @ widen(inp.W_ekn[int(inp.topk_ids[t, s])])
        assert np.max(np.abs(Y[p] - want)) <= 1e-12
    rows = np.array([5, 0, 100])
    assert np.array_equal(oracle.moe_gemm(inp.shards, inp.W_ekn, inp.topk_ids, rows=rows), Y[rows])


def test_moe_integer_inputs_exact():
    inp = wl.make_moe(wl.MOE_TINY, x_dist=("int", 2), w_dist=("int", 2))
    sh = inp.shape
    X = np.concatenate([widen(s) for s in inp.shards]).astype(np.int64)
    Y = oracle.moe_gemm(inp.shards, inp.W_ekn, inp.topk_ids)
    tok, slot, seg = oracle.moe_route(inp.topk_ids, sh.E)
    for e in range(sh.E):
        want = X[tok[seg[e]:seg[e + 1]]] @ widen(inp.W_ekn[e]).astype(np.int64)
        assert np.array_equal(Y[seg[e]:seg[e + 1]], want.astype(np.float64))


# ----------------------------------------------------------------------------------------------------------------
# MoE + ReduceScatter (Section 4.1, "MoE ReduceScatter"): grouped GEMM, top-k reduction, reduce scatter
# ----------------------------------------------------------------------------------------------------------------

def _moe_rs_by_hand(inp, W, rank):
    """The three steps written out with Python sorting and numpy fp64 products, sharing nothing with the oracle."""
    sh = inp.shape
    T, topk = inp.topk_ids.shape
    pairs = sorted((int(inp.topk_ids[t, s]), t, s) for t in range(T) for s in range(topk))     # (expert, token, slot)
    pos = {(t, s): p for p, (_, t, s) in enumerate(pairs)}
    H = wl.bf16_bits_to_f32(inp.H).astype(np.float64)
    W2 = wl.bf16_bits_to_f32(inp.W2_ekn).astype(np.float64)
    Tr = T // W
    R = np.zeros((Tr, sh.N))
    for i in range(Tr):
        t = rank * Tr + i
        for s in range(topk):
            e = int(inp.topk_ids[t, s])
            R[i] += float(inp.gate[t, s]) * (H[pos[(t, s)]] @ W2[e])
        for w in range(W):
            if w != rank:
                R[i] += inp.peer_slots[w][i].astype(np.float64)
    return R


@pytest.mark.parametrize("rank", [0, 3])
def test_moe_rs_oracle_against_steps_written_by_hand(rank):
    inp = wl.make_moe_rs(wl.MOE_RS_TINY, rank=rank)
    got = oracle.moe_rs(inp.H, inp.W2_ekn, inp.topk_ids, inp.gate, inp.peer_slots, wl.MOE_RS_TINY.W, rank)
    want = _moe_rs_by_hand(inp, wl.MOE_RS_TINY.W, rank)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)
    rows = np.array([5, 0, 23])
    sub = oracle.moe_rs(inp.H, inp.W2_ekn, inp.topk_ids, inp.gate, inp.peer_slots, wl.MOE_RS_TINY.W, rank, rows=rows)
    assert np.array_equal(sub, got[rows])


def test_moe_rs_special_cases():
    sh = wl.MoeRsShape("t", 17, 2, 6, 64, 8, 3, 2)
    inp = wl.make_moe_rs(sh, rank=0, h_dist=("int", 2), w_dist=("int", 2))
    zero = {1: np.zeros((sh.tokens_per_rank, sh.N), dtype=np.float32)}
    H = wl.bf16_bits_to_f32(inp.H).astype(np.float64)
    # (1) every expert holds the same matrix: the routing cancels and R = (sum_s gate * H[pos]) . W, one plain product
    same = np.repeat(inp.W2_ekn[:1], sh.E, axis=0)
    got = oracle.moe_rs(inp.H, same, inp.topk_ids, inp.gate, zero, sh.W, 0)
    tok, slot, seg = oracle.moe_route(inp.topk_ids, sh.E)
    mixed = np.zeros((sh.T, sh.Kl))
    for p in range(sh.T * sh.topk):
        mixed[tok[p]] += float(inp.gate[tok[p], slot[p]]) * H[p]
    want = mixed[: sh.tokens_per_rank] @ wl.bf16_bits_to_f32(same[0]).astype(np.float64)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)
    # (2) linear in the gate, and the peers' slices enter once each
    g2 = (inp.gate * np.float32(4.0)).astype(np.float32)        # a power of two: exact in float
    a = oracle.moe_rs(inp.H, inp.W2_ekn, inp.topk_ids, inp.gate, zero, sh.W, 0)
    b = oracle.moe_rs(inp.H, inp.W2_ekn, inp.topk_ids, g2, zero, sh.W, 0)
    assert np.allclose(b, 4.0 * a, rtol=1e-12, atol=1e-12)
    c = oracle.moe_rs(inp.H, inp.W2_ekn, inp.topk_ids, inp.gate, inp.peer_slots, sh.W, 0)
    assert np.allclose(c - a, inp.peer_slots[1].astype(np.float64), rtol=0, atol=1e-9)
    # (3) gate 1 on slot 0 and 0 on slot 1, integer data: R is row pos(t, 0) of the grouped GEMM, exactly
    g01 = np.zeros_like(inp.gate); g01[:, 0] = 1.0
    d = oracle.moe_rs(inp.H, inp.W2_ekn, inp.topk_ids, g01, zero, sh.W, 0)
    pos0 = {int(tok[p]): p for p in range(sh.T * sh.topk) if slot[p] == 0}
    for t in range(sh.tokens_per_rank):
        e = int(inp.topk_ids[t, 0])
        row = H[pos0[t]].astype(np.int64) @ wl.bf16_bits_to_f32(inp.W2_ekn[e]).astype(np.int64)
        assert np.array_equal(d[t], row.astype(np.float64))
    # (4) argument checks
    with pytest.raises(Exception):
        oracle.moe_rs(inp.H, inp.W2_ekn, inp.topk_ids, inp.gate, zero, 4, 0)          # T not a multiple of W

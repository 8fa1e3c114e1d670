"""Pins for the CPU oracle's AllGather and GEMM (no GPU).

Each test checks the oracle against something other than itself: a hand-worked
fixture, exact rational arithmetic, numpy's integer and fp64 matmul on the
special cases that reduce to them, closed forms and invariants.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(name):
    out = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *v = line.split()
            out[k] = [float(x) for x in v]
    return out


def bits(x):
    return wl.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def widen(b):
    return wl.bf16_bits_to_f32(b).astype(np.float64)


# ------------------------------------------------------------------ bf16


def test_bf16_rne_hand_values():
    # 1 + 2^-8 is a tie between 0x3F80 and 0x3F81 -> even (0x3F80); 1 + 3*2^-8 ties up to 0x3F82.
    assert oracle.f32_to_bf16(1.0) == 0x3F80
    assert oracle.f32_to_bf16(1.0 + 2.0**-8) == 0x3F80
    assert oracle.f32_to_bf16(1.0 + 3 * 2.0**-8) == 0x3F82
    assert oracle.f32_to_bf16(1.0 + 2.0**-8 + 2.0**-16) == 0x3F81
    assert oracle.f32_to_bf16(-2.5) == 0xC020
    assert oracle.f32_to_bf16(0.0) == 0x0000
    # largest finite fp32 rounds up to +Inf in bf16
    assert oracle.f32_to_bf16(np.finfo(np.float32).max) == 0x7F80
    assert oracle.bf16_to_f64(0x3F80) == 1.0 and oracle.bf16_to_f64(0xC020) == -2.5


def test_bf16_rne_matches_library_rounding():
    rng = np.random.default_rng(11)
    x = np.concatenate([rng.standard_normal(4000).astype(np.float32) * 37.0,
                        rng.uniform(-1, 1, 4000).astype(np.float32) * 1e-3])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.f32_to_bf16(v) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want)
    # the shared input generator quantises the same way
    assert np.array_equal(wl.f32_to_bf16_bits(x), want)


# -------------------------------------------------------------- allgather


@pytest.mark.parametrize("rank", [0, 1, 2])
def test_allgather_layout_is_rank_offset(rank):
    # Algorithm 2: rank r's shard lands at offset r*|L| whatever the calling rank is.
    W, Ms, K = 3, 4, 5
    shards = [bits(np.full((Ms, K), s + 1.0)) for s in range(W)]
    T = widen(oracle.allgather(shards, rank))
    for s in range(W):
        assert np.all(T[s * Ms:(s + 1) * Ms] == s + 1.0)


# ------------------------------------------------------------------- GEMM


def test_hand_worked_w2():
    g = _read_golden("ag_gemm_w2_2x2x2.txt")
    shards = [bits([g["shard0"]]), bits([g["shard1"]])]
    B = bits(np.array(g["B"]).reshape(2, 2))
    want = np.array(g["C"]).reshape(2, 2)
    for rank in (0, 1):
        assert np.array_equal(oracle.ag_gemm(shards, B, rank), want)


def test_exact_rational_brute_force():
    # bf16 values are dyadic rationals: Fraction arithmetic gives the exact product matrix.
    rng = np.random.default_rng(5)
    W, Ms, K, N = 2, 3, 7, 5
    shards = [bits(rng.uniform(-1, 1, (Ms, K))) for _ in range(W)]
    B = bits(rng.uniform(-1, 1, (K, N)))
    A = np.concatenate([widen(s) for s in shards])
    Bd = widen(B)
    got = oracle.ag_gemm(shards, B, 1)
    for i in range(W * Ms):
        for j in range(N):
            exact = sum(Fraction(A[i, k]) * Fraction(Bd[k, j]) for k in range(K))
            assert abs(Fraction(got[i, j]) - exact) <= abs(exact) * Fraction(1, 10**14) + Fraction(1, 10**15)


def test_w1_is_plain_gemm_vs_numpy():
    rng = np.random.default_rng(6)
    M, K, N = 37, 129, 53          # non-square: a transposed operand cannot pass
    A = bits(rng.uniform(-1, 1, (M, K)))
    B = bits(rng.standard_normal((K, N)) * 0.02)
    want = widen(A) @ widen(B)
    got = oracle.ag_gemm([A], B, 0)
    assert got.shape == (M, N)
    assert np.max(np.abs(got - want)) <= 1e-13 * np.sqrt(K)
    assert np.array_equal(got, oracle.gemm(A, B))


def test_integer_inputs_match_integer_matmul_exactly():
    inp = wl.make_ag_gemm(wl.AG_RAGGED, a_dist=("int", 2), b_dist=("int", 2))
    A = np.concatenate([widen(s) for s in inp.shards]).astype(np.int64)
    B = widen(inp.B_kn).astype(np.int64)
    want = A @ B                   # exact integer arithmetic
    for rank in range(inp.shape.W):
        got = oracle.ag_gemm(inp.shards, inp.B_kn, rank)
        assert np.array_equal(got, want.astype(np.float64))


def test_identity_b_returns_gathered_a():
    W, Ms, K = 4, 8, 32
    rng = np.random.default_rng(7)
    shards = [bits(rng.uniform(-1, 1, (Ms, K))) for _ in range(W)]
    eye = bits(np.eye(K))
    got = oracle.ag_gemm(shards, eye, 2)
    assert np.array_equal(got, np.concatenate([widen(s) for s in shards]))


def test_closed_forms():
    W, Ms, K, N = 4, 16, 96, 24
    ones = bits(np.ones((K, N)))
    # all ones: every output is K
    got = oracle.ag_gemm([bits(np.ones((Ms, K)))] * W, ones, 0)
    assert np.all(got == K)
    # shard s filled with s+1: rows of shard s equal (s+1)*K -- catches a misplaced or rotated shard
    shards = [bits(np.full((Ms, K), s + 1.0)) for s in range(W)]
    for rank in range(W):
        got = oracle.ag_gemm(shards, ones, rank)
        for s in range(W):
            assert np.all(got[s * Ms:(s + 1) * Ms] == (s + 1) * K)
    # a single 1 at A[i0,k0] selects row k0 of B into row i0 of C (index/sign/transposition check)
    rng = np.random.default_rng(8)
    B = bits(rng.uniform(-1, 1, (K, N)))
    A = np.zeros((W * Ms, K), dtype=np.float32)
    A[37, 11] = 1.0
    got = oracle.ag_gemm([bits(A[s * Ms:(s + 1) * Ms]) for s in range(W)], B, 0)
    want = np.zeros((W * Ms, N))
    want[37] = widen(B)[11]
    assert np.array_equal(got, want)


def test_linearity_on_integer_inputs():
    rng = np.random.default_rng(9)
    W, Ms, K, N = 2, 8, 64, 16
    shards = [bits(rng.integers(-3, 4, (Ms, K))) for _ in range(W)]
    B1 = rng.integers(-3, 4, (K, N)).astype(np.float32)
    B2 = rng.integers(-3, 4, (K, N)).astype(np.float32)
    lhs = oracle.ag_gemm(shards, bits(B1 + B2), 0)
    rhs = oracle.ag_gemm(shards, bits(B1), 0) + oracle.ag_gemm(shards, bits(B2), 0)
    assert np.array_equal(lhs, rhs)


def test_row_selection_matches_full_result():
    inp = wl.make_ag_gemm(wl.AG_TINY)
    full = oracle.ag_gemm(inp.shards, inp.B_kn, 0)
    rows = np.array([255, 0, 64, 63, 130], dtype=np.int64)
    assert np.array_equal(oracle.ag_gemm(inp.shards, inp.B_kn, 0, rows=rows), full[rows])


def test_rank_does_not_change_the_result():
    # The oracle has no notion of arrival order or of which shard is local.
    inp = wl.make_ag_gemm(wl.AG_TINY)
    ref = oracle.ag_gemm(inp.shards, inp.B_kn, 0)
    for rank in range(1, inp.shape.W):
        assert np.array_equal(oracle.ag_gemm(inp.shards, inp.B_kn, rank), ref)


def test_fp64_error_bound_against_exact_sum():
    # Error of the fp64 k-sum is far below the GPU tolerance: |err| <= K * 2^-53 * sum|a||b|.
    inp = wl.make_ag_gemm(wl.AG_TINY)
    A = np.concatenate([widen(s) for s in inp.shards])
    B = widen(inp.B_kn)
    got = oracle.ag_gemm(inp.shards, inp.B_kn, 0)
    import math
    for (i, j) in [(0, 0), (100, 200), (255, 255), (64, 1)]:
        exact = math.fsum(A[i, k] * B[k, j] for k in range(A.shape[1]))   # products are exact in fp64
        bound = A.shape[1] * 2.0**-53 * float(np.sum(np.abs(A[i]) * np.abs(B[:, j])))
        assert abs(got[i, j] - exact) <= bound


def test_invalid_arguments_are_rejected():
    A = bits(np.ones((4, 4)))
    with pytest.raises(ValueError):
        oracle.ag_gemm([A], A, 0, rows=np.array([4]))
    with pytest.raises(ValueError):
        oracle.allgather([A, A], 2)

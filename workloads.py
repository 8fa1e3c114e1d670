"""Seeded synthetic inputs for the AllGather-GEMM / GEMM-ReduceScatter hot path.

This module is shared by the CPU oracle's tests and by the HIP path's tests and
bench.  It holds input generation only: seeded draws, quantisation of the draws
to bf16 bit patterns, and the shape tables of the five workloads.  None of the
method's arithmetic (gather, GEMM, reduction, routing sort) lives here.

The paper's AG+GEMM / GEMM+RS shapes were printed only in figures (Section 4.1,
Section 4.3); the shapes here are LLM-MLP-shaped stand-ins, and the MoE shape
follows the style of Table 4 (tokens per rank, hidden sizes, experts, top-k).
All values are synthetic; no dataset or trained weight is involved.

Generator: numpy PCG64 (`numpy.random.default_rng(seed)`), fp32 draw, then
round-to-nearest-even to bf16.  seed = 1000 * cfg + stream id, with stream ids
A-shard s -> s, B -> 100, reduce-scatter peer slot w -> 200 + w, routing -> 300.
"""
from __future__ import annotations

import itertools
from dataclasses import dataclass, field

import numpy as np

# ----------------------------------------------------------------------------
# bf16 bit-pattern helpers (input quantisation only)
# ----------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 (nearest, ties to even); returns uint16 bit patterns.

    Inputs must be finite (the generators never draw NaN/Inf).
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = u + np.uint32(0x7FFF) + lsb
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to the fp32 values they denote (exact)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _seed(cfg: int, stream: int) -> int:
    return 1000 * cfg + stream


def _draw(rng: np.random.Generator, shape, dist: str, scale: float) -> np.ndarray:
    if dist == "uniform":          # U[-scale, scale)
        return rng.uniform(-scale, scale, size=shape).astype(np.float32)
    if dist == "normal":           # N(0, scale)
        return (rng.standard_normal(size=shape, dtype=np.float32) * np.float32(scale))
    if dist == "int":              # integers in {-scale..scale}: every fp32 partial sum is exact
        s = int(scale)
        return rng.integers(-s, s + 1, size=shape).astype(np.float32)
    if dist == "ones":
        return np.ones(shape, dtype=np.float32)
    raise ValueError(f"unknown distribution {dist!r}")


# ----------------------------------------------------------------------------
# AllGather-GEMM
# ----------------------------------------------------------------------------

@dataclass(frozen=True)
class AgGemmShape:
    """One rank's share of C = gather(A_0..A_{W-1}) . B_local."""
    name: str
    cfg: int            # seed namespace
    W: int              # world size (emulated)
    Ms: int             # rows per shard
    K: int
    N: int              # this rank's column share
    a_dist: tuple = ("uniform", 1.0)
    b_dist: tuple = ("uniform", 1.0)
    out: str = "bf16"   # dtype of C the workload names ("f32" or "bf16")

    @property
    def M(self) -> int:
        return self.W * self.Ms

    @property
    def flops(self) -> int:
        return 2 * self.M * self.N * self.K


AG_TINY = AgGemmShape("ag_gemm_tiny", 1, 4, 64, 256, 256, out="f32")
AG_8B = AgGemmShape("ag_gemm_8b_mlp", 2, 8, 512, 4096, 3584)
AG_70B = AgGemmShape("ag_gemm_70b_mlp", 3, 8, 1024, 8192, 7168, b_dist=("normal", 0.02))
# a mid-size shape with ragged M/N tails relative to any 128/256 tiling, for parity tests
AG_RAGGED = AgGemmShape("ag_gemm_ragged", 6, 3, 200, 320, 328, out="f32")

AG_SHAPES = {s.name: s for s in (AG_TINY, AG_8B, AG_70B, AG_RAGGED)}


@dataclass
class AgGemmInputs:
    shape: AgGemmShape
    shards: list        # W arrays [Ms, K] uint16 (bf16 bits); shards[s] lives on "rank" s
    B_kn: np.ndarray    # [K, N] uint16 (bf16 bits), logical K x N, row-major


def make_ag_gemm(shape: AgGemmShape, a_dist=None, b_dist=None) -> AgGemmInputs:
    a_dist = a_dist or shape.a_dist
    b_dist = b_dist or shape.b_dist
    shards = []
    for s in range(shape.W):
        rng = np.random.default_rng(_seed(shape.cfg, s))
        shards.append(f32_to_bf16_bits(_draw(rng, (shape.Ms, shape.K), *a_dist)))
    rng = np.random.default_rng(_seed(shape.cfg, 100))
    B = f32_to_bf16_bits(_draw(rng, (shape.K, shape.N), *b_dist))
    return AgGemmInputs(shape, shards, B)


def arrival_orders(W: int, rank: int, limit: int | None = None, seed: int = 0):
    """Orders in which the W-1 remote shards 'arrive' (lists of source ranks).

    All (W-1)! permutations if limit is None or they number at most `limit`;
    otherwise `limit` seeded random permutations, the rotated order first.
    """
    remotes = [(rank + j) % W for j in range(1, W)]
    n_all = 1
    for i in range(2, W):
        n_all *= i
    if limit is None or n_all <= limit:
        return [list(p) for p in itertools.permutations(remotes)]
    rng = np.random.default_rng(seed)
    out = [list(remotes)]
    while len(out) < limit:
        out.append([int(x) for x in rng.permutation(remotes)])
    return out


# ----------------------------------------------------------------------------
# GEMM-ReduceScatter
# ----------------------------------------------------------------------------

@dataclass(frozen=True)
class GemmRsShape:
    """Local partial GEMM [M, Kl] x [Kl, N] and the sum of this rank's row slice
    over W partial buffers (W-1 of them emulated peers)."""
    name: str
    cfg: int
    W: int
    M: int
    Kl: int
    N: int
    a_dist: tuple = ("uniform", 1.0)
    b_dist: tuple = ("normal", 0.02)
    slot_dist: tuple = ("normal", 1.0)

    @property
    def Ms(self) -> int:
        return self.M // self.W

    @property
    def gemm_flops(self) -> int:
        return 2 * self.M * self.N * self.Kl

    @property
    def reducer_bytes(self) -> int:
        """Compulsory HBM bytes of the reducer: W fp32 slices read, one written."""
        return (self.W + 1) * self.Ms * self.N * 4


RS_FULL = GemmRsShape("gemm_rs_full", 4, 8, 8192, 3584, 8192)
RS_TINY = GemmRsShape("gemm_rs_tiny", 7, 4, 256, 128, 192)
RS_SHAPES = {s.name: s for s in (RS_FULL, RS_TINY)}


@dataclass
class GemmRsInputs:
    shape: GemmRsShape
    A_loc: np.ndarray   # [M, Kl] uint16 bf16 bits
    B_kn: np.ndarray    # [Kl, N] uint16 bf16 bits
    peer_slots: dict    # w -> [Ms, N] float32 for every w != rank


def make_gemm_rs(shape: GemmRsShape, rank: int = 0, a_dist=None, b_dist=None,
                 slot_dist=None, with_gemm: bool = True) -> GemmRsInputs:
    a_dist = a_dist or shape.a_dist
    b_dist = b_dist or shape.b_dist
    slot_dist = slot_dist or shape.slot_dist
    A = B = None
    if with_gemm:
        rng = np.random.default_rng(_seed(shape.cfg, 0))
        A = f32_to_bf16_bits(_draw(rng, (shape.M, shape.Kl), *a_dist))
        rng = np.random.default_rng(_seed(shape.cfg, 100))
        B = f32_to_bf16_bits(_draw(rng, (shape.Kl, shape.N), *b_dist))
    slots = {}
    for w in range(shape.W):
        if w == rank:
            continue
        rng = np.random.default_rng(_seed(shape.cfg, 200 + w))
        slots[w] = _draw(rng, (shape.Ms, shape.N), *slot_dist)
    return GemmRsInputs(shape, A, B, slots)


# ----------------------------------------------------------------------------
# MoE AllGather grouped GEMM
# ----------------------------------------------------------------------------

@dataclass(frozen=True)
class MoeShape:
    """Tokens gathered from W shards, each routed to `topk` distinct experts;
    per-expert GEMM [rows_e, K] x [K, N] (tensor-parallel N slice)."""
    name: str
    cfg: int
    W: int
    tokens_per_rank: int
    K: int              # in hidden
    N: int              # out hidden (this rank's slice)
    E: int              # experts
    topk: int
    x_dist: tuple = ("uniform", 1.0)
    w_dist: tuple = ("normal", 0.02)

    @property
    def T(self) -> int:
        return self.W * self.tokens_per_rank

    @property
    def flops(self) -> int:
        return 2 * self.T * self.topk * self.K * self.N


MOE_FULL = MoeShape("ag_moe_full", 5, 8, 1024, 4096, 2048, 64, 2)
MOE_TINY = MoeShape("ag_moe_tiny", 8, 4, 48, 128, 96, 6, 2)
MOE_SHAPES = {s.name: s for s in (MOE_FULL, MOE_TINY)}


@dataclass
class MoeInputs:
    shape: MoeShape
    shards: list          # W arrays [tokens_per_rank, K] uint16 bf16 bits
    W_ekn: np.ndarray     # [E, K, N] uint16 bf16 bits (logical K x N per expert)
    topk_ids: np.ndarray  # [T, topk] int32, distinct experts per token


def make_moe(shape: MoeShape, x_dist=None, w_dist=None) -> MoeInputs:
    x_dist = x_dist or shape.x_dist
    w_dist = w_dist or shape.w_dist
    shards = []
    for s in range(shape.W):
        rng = np.random.default_rng(_seed(shape.cfg, s))
        shards.append(f32_to_bf16_bits(_draw(rng, (shape.tokens_per_rank, shape.K), *x_dist)))
    rng = np.random.default_rng(_seed(shape.cfg, 100))
    Wt = np.empty((shape.E, shape.K, shape.N), dtype=np.uint16)
    for e in range(shape.E):
        Wt[e] = f32_to_bf16_bits(_draw(rng, (shape.K, shape.N), *w_dist))
    rng = np.random.default_rng(_seed(shape.cfg, 300))
    # `topk` distinct experts per token, uniform: rank E uniform keys per token, take the smallest.
    keys = rng.random((shape.T, shape.E), dtype=np.float32)
    ids = np.argsort(keys, axis=1, kind="stable")[:, : shape.topk].astype(np.int32)
    return MoeInputs(shape, shards, Wt, np.ascontiguousarray(ids))


# ----------------------------------------------------------------------------
# MoE + ReduceScatter (second MoE layer, tensor parallel over K)
# ----------------------------------------------------------------------------

@dataclass(frozen=True)
class MoeRsShape:
    """T = W * tokens_per_rank tokens, each routed to `topk` distinct experts; rows of H are the (token, slot) pairs in
    routing order; per-expert GEMM [rows_e, Kl] x [Kl, N] (this rank's K slice), top-k weighted sum per token, then the
    sum over ranks of this rank's token slice."""
    name: str
    cfg: int
    W: int
    tokens_per_rank: int
    Kl: int             # in hidden / W
    N: int              # out hidden
    E: int
    topk: int
    h_dist: tuple = ("uniform", 1.0)
    w_dist: tuple = ("normal", 0.02)
    slot_dist: tuple = ("normal", 0.2)

    @property
    def T(self) -> int:
        return self.W * self.tokens_per_rank

    @property
    def flops(self) -> int:
        return 2 * self.T * self.topk * self.Kl * self.N


@dataclass
class MoeRsInputs:
    shape: MoeRsShape
    H: np.ndarray          # [T*topk, Kl] uint16 bf16 bits, rows in routing order
    W2_ekn: np.ndarray     # [E, Kl, N] uint16 bf16 bits
    topk_ids: np.ndarray   # [T, topk] int32
    gate: np.ndarray       # [T, topk] float32, positive, rows sum to 1
    peer_slots: dict       # w -> [tokens_per_rank, N] float32 for every w != rank


# Table 5, "MoE-RS-3": 1024 tokens per rank, in hidden 1536 (192 per rank at W = 8), out hidden 2048, 64 experts, top 2
MOE_RS_FULL = MoeRsShape("moe_rs_full", 15, 8, 1024, 192, 2048, 64, 2)
MOE_RS_TINY = MoeRsShape("moe_rs_tiny", 16, 4, 24, 64, 72, 5, 2)


def make_moe_rs(shape: MoeRsShape, rank: int = 0, h_dist=None, w_dist=None, slot_dist=None) -> MoeRsInputs:
    h_dist = h_dist or shape.h_dist
    w_dist = w_dist or shape.w_dist
    slot_dist = slot_dist or shape.slot_dist
    rng = np.random.default_rng(_seed(shape.cfg, 0))
    H = f32_to_bf16_bits(_draw(rng, (shape.T * shape.topk, shape.Kl), *h_dist))
    rng = np.random.default_rng(_seed(shape.cfg, 100))
    W2 = np.empty((shape.E, shape.Kl, shape.N), dtype=np.uint16)
    for e in range(shape.E):
        W2[e] = f32_to_bf16_bits(_draw(rng, (shape.Kl, shape.N), *w_dist))
    rng = np.random.default_rng(_seed(shape.cfg, 300))
    keys = rng.random((shape.T, shape.E), dtype=np.float32)
    ids = np.argsort(keys, axis=1, kind="stable")[:, : shape.topk].astype(np.int32)
    g = rng.random((shape.T, shape.topk), dtype=np.float32) + np.float32(0.1)
    gate = (g / g.sum(axis=1, keepdims=True)).astype(np.float32)
    slots = {}
    for w in range(shape.W):
        if w == rank:
            continue
        rng = np.random.default_rng(_seed(shape.cfg, 200 + w))
        slots[w] = _draw(rng, (shape.tokens_per_rank, shape.N), *slot_dist)
    return MoeRsInputs(shape, H, W2, np.ascontiguousarray(ids), gate, slots)

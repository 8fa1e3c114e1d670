/*
 * CPU oracle for the AllGather-GEMM consumer, the GEMM-ReduceScatter reducer and
 * the MoE AllGather grouped GEMM.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the plain definition of what the hot path
 * computes, written to be checked against the paper by eye: no tiling, no fusion,
 * no reordering.  It shares no code with the HIP path and is called only by the
 * tests, by the smoke check and by the bench's cpu_baseline leg.
 *
 * The overlapped method changes when each tile is computed, never what is
 * computed, so the oracle is the definition:
 *   - AllGather (Algorithm 2, pull mode): rank r's local buffer L_r lands at
 *     offset r * |L| of the symmetric buffer T.
 *   - AG+GEMM (Section 2.3, Figure 4): C = T . B with T viewed as [W*Ms, K].
 *   - ReduceScatter reduction (Algorithm 3, stream 2): R = sum over r = 0..W-1
 *     of T[r * |R| ...], in that order.
 *   - AG+MoE (Section 4.1, Table 4): a grouped GEMM over expert segments of the
 *     gathered tokens.
 *   - MoE+RS (Section 4.1, Table 5): grouped GEMM on the routed rows, top-k
 *     weighted reduction per token, sum of the ranks' partial slices.
 * Inputs are bf16 bit patterns; products and sums are taken in fp64 (a bf16 x bf16
 * product is exact in fp64, so only the additions round).  The one fp32 routine
 * (oracle_rs_reduce_f32) exists because the reducer's precision is fixed to fp32
 * by the build's contract and its summation order by Algorithm 3.
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -shared -fPIC (see oracle/build.py).
 * Every function returns 0, or a negative value on an invalid argument.
 */
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ bf16 */

static double bf16_bits_to_f64(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* fp32 -> bf16, round to nearest, ties to even.  NaN keeps a quiet-NaN pattern. */
uint16_t oracle_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t low = u & 0xffffu;          /* the 16 bits that are dropped */
    uint32_t keep = u >> 16;
    if (low > 0x8000u || (low == 0x8000u && (keep & 1u)))
        keep += 1u;                      /* carries into the exponent correctly; may reach Inf */
    return (uint16_t)keep;
}

double oracle_bf16_to_f64(uint16_t h) { return bf16_bits_to_f64(h); }

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------- AllGather */

/*
 * Algorithm 2 seen from `rank`: first the local copy T[rank*|L|] = L_rank, then,
 * for every other r, T[r*|L|] = (T at rank r)[r*|L|], which is L_r.
 * local_bufs[r] is rank r's local buffer L_r (shard_elems bf16 each);
 * T receives W * shard_elems bf16.
 */
int oracle_allgather(int W, int rank, int64_t shard_elems,
                     const uint16_t* const* local_bufs, uint16_t* T)
{
    if (W < 1 || rank < 0 || rank >= W || shard_elems < 0 || !local_bufs || !T)
        return -1;
    memcpy(T + (size_t)rank * shard_elems, local_bufs[rank], (size_t)shard_elems * 2);
    for (int r = 0; r < W; ++r) {
        if (r == rank)
            continue;
        memcpy(T + (size_t)r * shard_elems, local_bufs[r], (size_t)shard_elems * 2);
    }
    return 0;
}

/* ------------------------------------------------------------------ GEMM */

/*
 * C[i, :] = sum_k A[row(i), k] * B[k, :] for i in [0, n_rows), in fp64.
 * A is [M, K] bf16 row-major, B is [K, N] bf16 row-major (logical K x N),
 * rows = NULL means row(i) = i.  C is [n_rows, N] fp64 row-major.
 * Loop order i, k, j; the k sum of each output runs k = 0..K-1.
 */
static int gemm_rows_f64(int64_t M, int64_t K, int64_t N,
                         const uint16_t* A, const uint16_t* B,
                         const int64_t* rows, int64_t n_rows, double* C)
{
    if (M < 0 || K < 0 || N < 0 || n_rows < 0 || !C || (K > 0 && N > 0 && !B) ||
        (n_rows > 0 && K > 0 && !A))
        return -1;
    for (int64_t i = 0; i < n_rows; ++i) {
        int64_t r = rows ? rows[i] : i;
        if (r < 0 || r >= M)
            return -2;
    }
    double* Bd = (double*)malloc(sizeof(double) * (size_t)(K * N > 0 ? K * N : 1));
    if (!Bd)
        return -3;
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < K; ++k)
        for (int64_t j = 0; j < N; ++j)
            Bd[k * N + j] = bf16_bits_to_f64(B[k * N + j]);

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < n_rows; ++i) {
        const int64_t r = rows ? rows[i] : i;
        double* c = C + i * N;
        for (int64_t j = 0; j < N; ++j)
            c[j] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const double a = bf16_bits_to_f64(A[r * K + k]);
            const double* b = Bd + k * N;
            for (int64_t j = 0; j < N; ++j)
                c[j] += a * b[j];
        }
    }
    free(Bd);
    return 0;
}

int oracle_gemm(int64_t M, int64_t K, int64_t N, const uint16_t* A, const uint16_t* B,
                const int64_t* rows, int64_t n_rows, double* C)
{
    return gemm_rows_f64(M, K, N, A, B, rows, n_rows, C);
}

/*
 * AllGather-GEMM for one rank: gather the W shards (each [Ms, K]) into T as
 * Algorithm 2 lays them out, then C = T . B on the selected rows of T
 * (rows index the gathered matrix, 0 <= row < W*Ms; NULL = all rows in order,
 * and then n_rows must be W*Ms).
 */
int oracle_ag_gemm(int W, int rank, int64_t Ms, int64_t K, int64_t N,
                   const uint16_t* const* shards, const uint16_t* B,
                   const int64_t* rows, int64_t n_rows, double* C)
{
    if (W < 1 || Ms < 0 || K < 0)
        return -1;
    const int64_t M = (int64_t)W * Ms;
    if (!rows && n_rows != M)
        return -1;
    uint16_t* T = (uint16_t*)malloc((size_t)(M * K > 0 ? M * K : 1) * 2);
    if (!T)
        return -3;
    int rc = oracle_allgather(W, rank, Ms * K, shards, T);
    if (rc == 0)
        rc = gemm_rows_f64(M, K, N, T, B, rows, n_rows, C);
    free(T);
    return rc;
}

/* ----------------------------------------------------------- ReduceScatter */

/* R[i] = sum_{w=0}^{W-1} T_w[i] in fp64 (the definition of the reduction). */
int oracle_rs_reduce_f64(int W, int64_t n, const float* const* slots, double* R)
{
    if (W < 1 || n < 0 || !slots || !R)
        return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double acc = 0.0;
        for (int w = 0; w < W; ++w)
            acc += (double)slots[w][i];
        R[i] = acc;
    }
    return 0;
}

/*
 * The same reduction with the precision and order the reducer is bound to:
 * R starts at +0 and takes R = R + T_w in fp32 for w = 0, 1, .., W-1
 * (the loop of Algorithm 3, stream 2).  Each addition rounds to fp32.
 */
int oracle_rs_reduce_f32(int W, int64_t n, const float* const* slots, float* R)
{
    if (W < 1 || n < 0 || !slots || !R)
        return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        volatile float acc = 0.0f;       /* volatile: one rounding per addition, no wider temporaries */
        for (int w = 0; w < W; ++w)
            acc = acc + slots[w][i];
        R[i] = acc;
    }
    return 0;
}

/*
 * GEMM + ReduceScatter for one rank: the local partial product
 * P = A_loc[M, Kl] . B_loc[Kl, N], of which only this rank's row slice
 * [rank*Ms, (rank+1)*Ms) takes part, plus the W-1 peers' partial slices
 * (given, fp32, [Ms, N] each; slots[rank] is ignored), summed in fp64.
 * rows index the slice (0 <= row < Ms; NULL = all, n_rows = Ms).
 * R is [n_rows, N] fp64.
 */
int oracle_gemm_rs(int W, int rank, int64_t M, int64_t Kl, int64_t N,
                   const uint16_t* A_loc, const uint16_t* B_loc,
                   const float* const* slots,
                   const int64_t* rows, int64_t n_rows, double* R)
{
    if (W < 1 || rank < 0 || rank >= W || M % W != 0)
        return -1;
    const int64_t Ms = M / W;
    if (!rows && n_rows != Ms)
        return -1;
    int64_t* grow = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n_rows > 0 ? n_rows : 1));
    if (!grow)
        return -3;
    for (int64_t i = 0; i < n_rows; ++i) {
        int64_t r = rows ? rows[i] : i;
        if (r < 0 || r >= Ms) {
            free(grow);
            return -2;
        }
        grow[i] = (int64_t)rank * Ms + r;
    }
    int rc = gemm_rows_f64(M, Kl, N, A_loc, B_loc, grow, n_rows, R);
    if (rc == 0) {
        for (int w = 0; w < W; ++w) {
            if (w == rank)
                continue;
            for (int64_t i = 0; i < n_rows; ++i) {
                const int64_t r = rows ? rows[i] : i;
                for (int64_t j = 0; j < N; ++j)
                    R[i * N + j] += (double)slots[w][r * N + j];
            }
        }
    }
    free(grow);
    return rc;
}

/* --------------------------------------------------------------------- MoE */

/*
 * Routing order: the (token, slot) pairs sorted by (expert, token, slot).
 * topk_ids is [T, topk]; pair_token / pair_expert receive T*topk entries in sorted
 * order; seg_off receives E+1 offsets (expert e owns sorted rows
 * [seg_off[e], seg_off[e+1])).  Written as the definition: one pass per expert.
 */
int oracle_moe_route(int64_t T, int topk, int E, const int32_t* topk_ids,
                     int32_t* pair_token, int32_t* pair_slot, int64_t* seg_off)
{
    if (T < 0 || topk < 1 || E < 1 || !topk_ids || !pair_token || !pair_slot || !seg_off)
        return -1;
    for (int64_t i = 0; i < T * topk; ++i)
        if (topk_ids[i] < 0 || topk_ids[i] >= E)
            return -2;
    int64_t p = 0;
    for (int e = 0; e < E; ++e) {
        seg_off[e] = p;
        for (int64_t t = 0; t < T; ++t)
            for (int s = 0; s < topk; ++s)
                if (topk_ids[t * topk + s] == e) {
                    pair_token[p] = (int32_t)t;
                    pair_slot[p] = s;
                    ++p;
                }
    }
    seg_off[E] = p;
    return p == T * topk ? 0 : -2;
}

/*
 * Y[i, :] = X[token(p_i), :] . W_{expert(p_i)} for the selected sorted rows p_i,
 * X = the gathered tokens [T, K] (shards laid out as in Algorithm 2),
 * Wt = [E, K, N] bf16.  rows index the sorted pair list (NULL = all T*topk rows).
 */
int oracle_moe_gemm(int W, int rank, int64_t tokens_per_rank, int64_t K, int64_t N, int E, int topk,
                    const uint16_t* const* shards, const uint16_t* Wt, const int32_t* topk_ids,
                    const int64_t* rows, int64_t n_rows, double* Y)
{
    if (W < 1 || tokens_per_rank < 0 || K < 0 || N < 0)
        return -1;
    const int64_t T = (int64_t)W * tokens_per_rank;
    const int64_t P = T * topk;
    if (!rows && n_rows != P)
        return -1;
    int rc = 0;
    uint16_t* X = (uint16_t*)malloc((size_t)(T * K > 0 ? T * K : 1) * 2);
    int32_t* ptok = (int32_t*)malloc(sizeof(int32_t) * (size_t)(P > 0 ? P : 1));
    int32_t* pslot = (int32_t*)malloc(sizeof(int32_t) * (size_t)(P > 0 ? P : 1));
    int64_t* seg = (int64_t*)malloc(sizeof(int64_t) * (size_t)(E + 1));
    if (!X || !ptok || !pslot || !seg) {
        rc = -3;
        goto done;
    }
    rc = oracle_allgather(W, rank, tokens_per_rank * K, shards, X);
    if (rc)
        goto done;
    rc = oracle_moe_route(T, topk, E, topk_ids, ptok, pslot, seg);
    if (rc)
        goto done;
    for (int64_t i = 0; i < n_rows; ++i) {
        int64_t p = rows ? rows[i] : i;
        if (p < 0 || p >= P) {
            rc = -2;
            goto done;
        }
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < n_rows; ++i) {
        const int64_t p = rows ? rows[i] : i;
        const int64_t t = ptok[p];
        const int e = topk_ids[t * topk + pslot[p]];
        const uint16_t* w = Wt + (size_t)e * K * N;
        double* y = Y + i * N;
        for (int64_t j = 0; j < N; ++j)
            y[j] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const double a = bf16_bits_to_f64(X[t * K + k]);
            for (int64_t j = 0; j < N; ++j)
                y[j] += a * bf16_bits_to_f64(w[k * N + j]);
        }
    }
done:
    free(X);
    free(ptok);
    free(pslot);
    free(seg);
    return rc;
}

/* -------------------------------------------------- MoE + ReduceScatter (Section 4.1) */

/*
 * MoE + ReduceScatter for one rank (Section 4.1, "MoE ReduceScatter": grouped GEMM, top-k reduction, reduce
 * scatter; tensor parallel over K), in the order of those three steps:
 *   Y[p, :]  = H[p, :] . W2_{expert(p)}          for every sorted pair p   (H is [T*topk, Kl], rows in routing order)
 *   Z[t, :]  = sum_s gate[t, s] * Y[pos(t, s), :]                          (pos = place of pair (t, s) in that order)
 *   R[i, :]  = Z[rank*Tr + i, :] + sum_{w != rank} slots[w][i, :]          (Tr = T / W tokens per rank)
 * W2t is [E, Kl, N] bf16 (logical K x N per expert), gate [T, topk] float, slots[w] float [Tr, N] (slots[rank]
 * unused).  rows selects tokens of the own slice (NULL = all Tr).
 */
int oracle_moe_rs(int W, int rank, int64_t T, int64_t Kl, int64_t N, int E, int topk,
                  const uint16_t* H, const uint16_t* W2t, const int32_t* topk_ids, const float* gate,
                  const float* const* slots, const int64_t* rows, int64_t n_rows, double* R)
{
    if (W < 1 || rank < 0 || rank >= W || T < 0 || T % W != 0 || Kl < 0 || N < 0 || topk < 1 || E < 1)
        return -1;
    if (!H || !W2t || !topk_ids || !gate || !slots || !R)
        return -1;
    const int64_t Tr = T / W, P = T * topk;
    if (!rows && n_rows != Tr)
        return -1;
    for (int w = 0; w < W; ++w)
        if (w != rank && !slots[w])
            return -1;
    int rc = 0;
    int32_t* ptok = (int32_t*)malloc(sizeof(int32_t) * (size_t)(P > 0 ? P : 1));
    int32_t* pslot = (int32_t*)malloc(sizeof(int32_t) * (size_t)(P > 0 ? P : 1));
    int64_t* pos = (int64_t*)malloc(sizeof(int64_t) * (size_t)(P > 0 ? P : 1));
    int64_t* seg = (int64_t*)malloc(sizeof(int64_t) * (size_t)(E + 1));
    if (!ptok || !pslot || !pos || !seg) {
        rc = -3;
        goto done;
    }
    rc = oracle_moe_route(T, topk, E, topk_ids, ptok, pslot, seg);
    if (rc)
        goto done;
    for (int64_t p = 0; p < P; ++p)
        pos[(int64_t)ptok[p] * topk + pslot[p]] = p;
    for (int64_t i = 0; i < n_rows; ++i) {
        const int64_t r = rows ? rows[i] : i;
        if (r < 0 || r >= Tr) {
            rc = -2;
            goto done;
        }
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < n_rows; ++i) {
        const int64_t r = rows ? rows[i] : i;
        const int64_t t = (int64_t)rank * Tr + r;
        double* out = R + i * N;
        double* y = (double*)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
        for (int64_t j = 0; j < N; ++j)
            out[j] = 0.0;
        for (int s = 0; s < topk; ++s) {
            const int64_t p = pos[t * topk + s];
            const int e = topk_ids[t * topk + s];
            const uint16_t* w2 = W2t + (size_t)e * Kl * N;
            for (int64_t j = 0; j < N; ++j)
                y[j] = 0.0;
            for (int64_t k = 0; k < Kl; ++k) {                       /* grouped GEMM row */
                const double a = bf16_bits_to_f64(H[p * Kl + k]);
                for (int64_t j = 0; j < N; ++j)
                    y[j] += a * bf16_bits_to_f64(w2[k * N + j]);
            }
            const double g = (double)gate[t * topk + s];            /* top-k reduction */
            for (int64_t j = 0; j < N; ++j)
                out[j] += g * y[j];
        }
        for (int w = 0; w < W; ++w)                                 /* reduce scatter: the peers' partial sums */
            if (w != rank)
                for (int64_t j = 0; j < N; ++j)
                    out[j] += (double)slots[w][r * N + j];
        free(y);
    }
done:
    free(ptok);
    free(pslot);
    free(pos);
    free(seg);
    return rc;
}

/*
 * Bandwidth (GB/s) the local reduction must sustain for perfect overlap in the
 * cross-node ReduceScatter analysis of Section 3.5: with volume B per slice, the
 * intra-node scatter takes (W-1) B / link, the P2P send B / nic, and the
 * reduction (reads W slices, writes one) must fit in the difference.
 */
double oracle_rs_required_bandwidth(int W, double link_GBps, double nic_GBps)
{
    const double t_left = (double)(W - 1) / link_GBps - 1.0 / nic_GBps; /* per unit volume */
    if (t_left <= 0.0)
        return -1.0;
    return (double)(W + 1) / t_left;
}

// Routing for the MoE AllGather grouped GEMM (Section 4.1, "AllGather MoE"): from the top-k expert ids of every
// token to the list of (token, slot) pairs sorted by (expert, token, slot), the expert segment offsets, and the
// table of output tiles the grouped GEMM walks.  Integer work only; every kernel is deterministic (no atomics
// decide a position).
#include "agg_internal.h"

namespace agg {

constexpr int kMaxExperts = 4096;     // histogram bins held in LDS

// One kernel, one workgroup per expert.  Every workgroup builds the full histogram of the ids in LDS (counts do not
// depend on the order of the atomic adds), takes its own segment offset and first tile index from the prefix sums,
// then writes the tokens of its expert's pairs in (token, slot) order -- the order of the flat pair index -- and
// the expert's tile entries.  Tiles of an expert are listed n-tile by n-tile, the m-tiles of one n-tile next to
// each other, so that the workgroups of one XCD (which take consecutive tiles) read the same rows of that
// expert's weights at the same time.  Workgroup 0 also writes the segment offsets and the tile count.
__global__ __launch_bounds__(256) void moe_route_kernel(const MoeRouteArgs a)
{
    const int e = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    extern __shared__ int hist[];                 // [E] counts
    __shared__ int wave_cnt[2][8][4];
    __shared__ int s_seg_lo, s_first;
    for (int i = tid; i < a.E; i += 256) hist[i] = 0;
    __syncthreads();
    // ---- pass 1: histogram (four ids per lane per step)
    const int4* ids4 = (const int4*)a.topk_ids;
    const int n4 = a.P / 4;
    for (int i = tid; i < n4; i += 256) {
        const int4 v = ids4[i];
        if ((unsigned)v.x < (unsigned)a.E) atomicAdd(&hist[v.x], 1);
        if ((unsigned)v.y < (unsigned)a.E) atomicAdd(&hist[v.y], 1);
        if ((unsigned)v.z < (unsigned)a.E) atomicAdd(&hist[v.z], 1);
        if ((unsigned)v.w < (unsigned)a.E) atomicAdd(&hist[v.w], 1);
    }
    for (int i = 4 * n4 + tid; i < a.P; i += 256) {
        const int v = a.topk_ids[i];
        if ((unsigned)v < (unsigned)a.E) atomicAdd(&hist[v], 1);
    }
    __syncthreads();
    // ---- prefix sums over the experts before e (wave 0; E is small)
    if (wave == 0) {
        int off = 0, tiles = 0;
        for (int i = lane; i < e; i += 64) {
            const int c = hist[i];
            off += c;
            tiles += ((c + a.bm - 1) / a.bm) * a.tiles_n;
        }
        for (int sft = 32; sft > 0; sft >>= 1) {
            off += __shfl_down(off, sft);
            tiles += __shfl_down(tiles, sft);
        }
        if (lane == 0) { s_seg_lo = off; s_first = tiles; }
    }
    __syncthreads();
    const int seg_lo = s_seg_lo, cnt = hist[e], seg_hi = seg_lo + cnt, first = s_first;
    if (e == a.E - 1 && tid == 0) {
        a.seg_off[a.E] = seg_hi;
        const int total = first + ((cnt + a.bm - 1) / a.bm) * a.tiles_n;
        *a.n_tiles_dev = total <= a.tab_capacity ? total : 0;   // the capacity is an upper bound by construction
    }
    if (tid == 0) a.seg_off[e] = seg_lo;

    // ---- pass 2: stable placement, 1024 pairs per step (lane handles 4 consecutive pairs), U steps per pass of the
    // loop: their ids are loaded together and their counts exchanged with one barrier, not one per step.
    constexpr int U = 8;
    int running = seg_lo;
    for (int base0 = 0; base0 < a.P; base0 += 1024 * U) {
      int vv[U][4];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int i0 = base0 + u * 1024 + 4 * tid;
        if (i0 + 3 < a.P && (a.P & 3) == 0) {
            const int4 q = ids4[i0 >> 2];
            vv[u][0] = q.x; vv[u][1] = q.y; vv[u][2] = q.z; vv[u][3] = q.w;
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) vv[u][k] = i0 + k < a.P ? a.topk_ids[i0 + k] : -1;
        }
      }
      // counts of this expert's pairs: per lane, then per wave, for all U steps; one barrier; then the positions
      int mine[U], incl[U];
      const int par = (base0 / (1024 * U)) & 1;       // wave_cnt is double-buffered over the passes of this loop
#pragma unroll
      for (int u = 0; u < U; ++u) {
        mine[u] = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) mine[u] += (vv[u][k] == e);
        // inclusive prefix of `mine` over the wave, in lane order
        incl[u] = mine[u];
#pragma unroll
        for (int sft = 1; sft < 64; sft <<= 1) {
            const int t = __shfl_up(incl[u], sft);
            if (lane >= sft) incl[u] += t;
        }
        if (lane == 63) wave_cnt[par][u][wave] = incl[u];
      }
      __syncthreads();
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int i0 = base0 + u * 1024 + 4 * tid;
        int before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const int c = wave_cnt[par][u][w];
            if (w < wave) before += c;
            total += c;
        }
        int pos = running + before + incl[u] - mine[u];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (vv[u][k] == e) {
                if (a.pair_pos) a.pair_pos[i0 + k] = pos;
                a.sorted_token[pos++] = (i0 + k) / a.topk;
            } else if (e == 0 && a.pair_pos && i0 + k < a.P && (unsigned)vv[u][k] >= (unsigned)a.E) {
                a.pair_pos[i0 + k] = -1;          // an id outside [0, E): the pair is nowhere in the sorted order
            }
        }
        running += total;
      }
    }
    // ---- tile entries (they read sorted_token written above by this same workgroup)
    __threadfence_block();
    __syncthreads();
    const int mt = (cnt + a.bm - 1) / a.bm;
    if (first + mt * a.tiles_n > a.tab_capacity) return;
    for (int k = tid; k < mt * a.tiles_n; k += 256) {
        const int n = k / mt, m = k - n * mt;
        MoeTile t;
        t.expert = e;
        t.m0 = seg_lo + m * a.bm;
        t.m_end = min(t.m0 + a.bm, seg_hi);
        t.n_tile = n;
        // tokens rise inside a segment: the first and last token bound the rows of T this tile reads
        const int tok_lo = a.sorted_token[t.m0], tok_hi = a.sorted_token[t.m_end - 1];
        t.f_lo = min(tok_lo / a.rows_per_flag, a.n_flags - 1);
        t.f_hi = min(tok_hi / a.rows_per_flag, a.n_flags - 1);
        t.st_lo = t.m0;
        t.st_hi = t.m_end;
        if (a.keep_lo < a.keep_hi) {
            // tokens rise inside the segment: the rows of tokens in [keep_lo, keep_hi) are one run of the tile's rows
            auto first_not_below = [&](int tok) {
                int lo = t.m0, hi = t.m_end;
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (a.sorted_token[mid] < tok) lo = mid + 1; else hi = mid;
                }
                return lo;
            };
            t.st_lo = first_not_below(a.keep_lo);
            t.st_hi = first_not_below(a.keep_hi);
        }
        a.tile_tab[first + k] = t;
    }
}

// Top-k reduction (Section 4.1, "MoE ReduceScatter", the step between the grouped GEMM and the reduce scatter):
// every token's `topk` rows of Y are weighted with its gate values and summed in slot order, fp32, starting from the
// first product.  Streaming: one float4 per lane, tokens of this rank first (their slice is what the reducer waits for).
__global__ __launch_bounds__(256) void topk_reduce_kernel(const TopkReduceArgs a)
{
    typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
    const int n4 = a.N / 4;
    const long long total = (long long)a.T * n4;
    const int own_n = a.own_hi - a.own_lo;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
        int v = (int)(i / n4);                       // place in the order: own tokens first, then the others
        const int j = (int)(i - (long long)v * n4);
        int t;
        if (v < own_n) t = a.own_lo + v;
        else { t = v - own_n; if (t >= a.own_lo) t += own_n; }
        const bool own = t >= a.own_lo && t < a.own_hi;
        if (!own && !a.Z_other) continue;
        f32x4 z = {0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < a.topk; ++s) {
            const int p = a.pair_pos[t * a.topk + s];
            if (p < 0) continue;                  // a pair with an invalid expert id contributes nothing
            const float g = a.gate[t * a.topk + s];
            const f32x4 y = __builtin_nontemporal_load((const f32x4*)(a.Y + (long long)p * a.N) + j);
            z = z + g * y;
        }
        f32x4* dst = own ? (f32x4*)(a.Z_own + (long long)(t - a.own_lo) * a.N) + j : (f32x4*)(a.Z_other + (long long)t * a.N) + j;
        *dst = z;
    }
}

hipError_t launch_topk_reduce(const TopkReduceArgs& a, int n_workgroups, hipStream_t stream)
{
    hipLaunchKernelGGL(topk_reduce_kernel, dim3(n_workgroups), dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_moe_route(const MoeRouteArgs& a, hipStream_t stream)
{
    if (a.E > kMaxExperts) return hipErrorInvalidValue;
    hipLaunchKernelGGL(moe_route_kernel, dim3(a.E), dim3(256), (size_t)a.E * sizeof(int), stream, a);
    return hipGetLastError();
}

}  // namespace agg

// Routing for the MoE AllGather grouped GEMM (Section 4.1, "AllGather MoE"): from the top-k expert ids of every
// token to the list of (token, slot) pairs sorted by (expert, token, slot), the expert segment offsets, and the
// table of output tiles the grouped GEMM walks.  Integer work only; every kernel is deterministic (no atomics
// decide a position).
#include "agg_internal.h"

namespace agg {

// Workgroup e counts the pairs routed to expert e.
__global__ __launch_bounds__(256) void moe_count_kernel(const MoeRouteArgs a)
{
    const int e = blockIdx.x, tid = threadIdx.x;
    int n = 0;
    for (int i = tid; i < a.P; i += 256) n += (a.topk_ids[i] == e);
    __shared__ int part[256];
    part[tid] = n;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (tid < s) part[tid] += part[tid + s];
        __syncthreads();
    }
    if (tid == 0) a.counts[e] = part[0];
}

// Segment offsets and, per expert, the index of its first tile.  Tiles of an expert are listed n-tile by n-tile,
// the m-tiles of one n-tile next to each other, so that the workgroups of one XCD (which take consecutive tiles)
// read the same rows of that expert's weights at the same time.
__global__ __launch_bounds__(256) void moe_prefix_kernel(const MoeRouteArgs a)
{
    if (threadIdx.x == 0) {
        int off = 0, tiles = 0;
        for (int e = 0; e < a.E; ++e) {
            a.seg_off[e] = off;
            a.tile_first[e] = tiles;
            const int c = a.counts[e];
            off += c;
            tiles += ((c + a.bm - 1) / a.bm) * a.tiles_n;
        }
        a.seg_off[a.E] = off;
        a.tile_first[a.E] = tiles;
        *a.n_tiles_dev = tiles <= a.tab_capacity ? tiles : 0;   // the capacity is an upper bound by construction
    }
}

// Workgroup e writes the tokens of expert e's pairs in (token, slot) order -- the order of the flat pair index --
// then the expert's tile entries.
__global__ __launch_bounds__(256) void moe_place_kernel(const MoeRouteArgs a)
{
    const int e = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    __shared__ int wave_cnt[4];
    const int seg_lo = a.seg_off[e], seg_hi = a.seg_off[e + 1];
    int running = seg_lo;
    for (int base = 0; base < a.P; base += 256) {
        const int i = base + tid;
        const bool match = i < a.P && a.topk_ids[i] == e;
        const unsigned long long bal = __ballot(match);
        if (lane == 0) wave_cnt[wave] = __popcll(bal);
        __syncthreads();
        int before = 0, total = 0;
        for (int w = 0; w < 4; ++w) {
            if (w < wave) before += wave_cnt[w];
            total += wave_cnt[w];
        }
        if (match) a.sorted_token[running + before + __popcll(bal & ((1ull << lane) - 1ull))] = i / a.topk;
        running += total;
        __syncthreads();
    }
    // tile entries (they read sorted_token written above by this same workgroup)
    __threadfence_block();
    __syncthreads();
    const int cnt = seg_hi - seg_lo;
    const int mt = (cnt + a.bm - 1) / a.bm;
    const int first = a.tile_first[e];
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
        t.pad0 = t.pad1 = 0;
        a.tile_tab[first + k] = t;
    }
}

hipError_t launch_moe_route(const MoeRouteArgs& a, hipStream_t stream)
{
    hipLaunchKernelGGL(moe_count_kernel, dim3(a.E), dim3(256), 0, stream, a);
    hipLaunchKernelGGL(moe_prefix_kernel, dim3(1), dim3(256), 0, stream, a);
    hipLaunchKernelGGL(moe_place_kernel, dim3(a.E), dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace agg

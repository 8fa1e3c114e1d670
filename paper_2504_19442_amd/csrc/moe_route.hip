// Routing for the MoE AllGather grouped GEMM (Section 4.1, "AllGather MoE"): from the top-k expert ids of every
// token to the list of (token, slot) pairs sorted by (expert, token, slot), the expert segment offsets, and the
// table of output tiles the grouped GEMM walks.  Integer work only; every kernel is deterministic (no atomics
// decide a position).
#include "agg_internal.h"

namespace agg {

constexpr int kSegTokLds = 2048;      // an expert's sorted tokens are kept in LDS for the tile entries up to this many
constexpr int kRouteWaves = 16, kRouteThreads = 64 * kRouteWaves;
constexpr int kRouteSteps = 4;
constexpr int kChunk = kRouteWaves * kRouteSteps * 256;     // pairs taken at a time: 16 waves x 4 steps x 64 lanes x 4 pairs

// One kernel, one workgroup per expert.  Only one pair in E belongs to the expert, so the work per pair is kept to a
// compare: a wave takes 1024 consecutive pairs of a chunk (a lane 4 consecutive ones in each of 4 steps), the place
// of a matching pair among the workgroup's matches comes from ballots and lane-mask bit counts, the matches are
// compacted into LDS as offsets inside the chunk, and only then turned into tokens and stored, one match per lane:
// the tokens of the expert's pairs in (token, slot) order -- the order of the flat pair index.
//
// The segment offset of an expert is the sum of the counts of the experts before it.  Every workgroup publishes its
// count in the control block and reads those of the experts before it (waiting for them where needed; it compacts
// its matches meanwhile).  A workgroup takes its expert from a ticket counter, not from its index in the grid: a
// workgroup that holds ticket e knows that the holders of the tickets below e are already running, so its wait ends
// whatever order the hardware starts workgroups in.  Counts are tagged with the number of the call (a device word
// that the holder of the last ticket advances, after which it puts the ticket counter back to zero): entries of earlier
// calls are never taken for this call's, nothing has to be cleared between calls, and a launch replayed from a HIP
// graph works like a fresh one.  Waits are bounded by the context's time limit like the GEMM's waits for signals.
//
// Tiles of an expert are listed n-tile by n-tile, the m-tiles of one n-tile next to each other, so that the
// workgroups of one XCD (which take consecutive tiles) read the same rows of that expert's weights at the same time.
__global__ __launch_bounds__(kRouteThreads) void moe_route_kernel(const MoeRouteArgs a)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    __shared__ int s_e, s_cnt[kRouteWaves], s_below[2][kRouteWaves], wave_tot[2][kRouteWaves], s_seg_lo, s_first;
    __shared__ unsigned s_tag;
    __shared__ int seg_tok[kSegTokLds];           // this expert's tokens in sorted order, while they fit
    __shared__ unsigned short cidx[kChunk];       // the chunk's matching pairs (offset inside the chunk), in order
    unsigned* const call_word = (unsigned*)(a.ctrl + kMoeCtrlCall);
    unsigned* const ticket_word = (unsigned*)(a.ctrl + kMoeCtrlTicket);
    unsigned long long* const counts = (unsigned long long*)(a.ctrl + kMoeCtrlCounts);
    unsigned long long* const kept = (unsigned long long*)(a.ctrl + kMoeCtrlKept);
    // keep_lo < keep_hi: only the rows of tokens in [keep_lo, keep_hi) get tiles.  Tokens rise inside a segment, so
    // they are one run of its rows: from the number of the expert's pairs below flat pair index keep_lo * topk to the
    // number below keep_hi * topk.
    const bool keep = a.keep_lo < a.keep_hi;
    const int x_lo = keep ? a.keep_lo * a.topk : 0, x_hi = keep ? a.keep_hi * a.topk : 0;
    // All loads of a chunk are issued before the first use: one memory latency per chunk.  When all pairs fit one
    // chunk, the placement works on the registers the count loaded.
    constexpr int U = kRouteSteps;
    const int4* ids4 = (const int4*)a.topk_ids;
    const int lane_off = wave * (kChunk / kRouteWaves) + 4 * lane;      // + u * 256: offset of this lane's 4 pairs of step u
    int vv[U][4];
    auto load_chunk = [&](int base0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i0 = base0 + lane_off + u * 256;
            if (i0 + 3 < a.P) {                      // (i0 is a multiple of 4: the 16-byte load is aligned)
                const int4 q = ids4[i0 >> 2];
                vv[u][0] = q.x; vv[u][1] = q.y; vv[u][2] = q.z; vv[u][3] = q.w;
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k) vv[u][k] = i0 + k < a.P ? a.topk_ids[i0 + k] : -1;
            }
        }
    };
    const bool one_chunk = a.P <= kChunk;
    load_chunk(0);
    if (tid == 0) {
        s_tag = __hip_atomic_load(call_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u;
        s_e = (int)__hip_atomic_fetch_add(ticket_word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    const int e = s_e;
    const unsigned tag = s_tag;
    if (e >= a.E) {                                  // the ticket counter was not at zero: an earlier call never finished
        if (tid == 0) *a.err = 1;
        return;
    }
    // matches of this wave in front of this lane's pairs of step u (earlier steps, and lower lanes of step u);
    // returns the wave's matches in the chunk (the same in every lane)
    int before[U];
    int below_lo = 0, below_hi = 0;                  // the wave's matches below x_lo / x_hi, over all chunks counted
    auto count_chunk = [&](int base0, bool with_bounds) {
        int wtot = 0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int b = wtot;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const bool hit = vv[u][k] == e;
                const unsigned long long m = __ballot(hit);
                b += __builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
                wtot += __popcll(m);
                if (with_bounds) {
                    const int i = base0 + lane_off + u * 256 + k;
                    below_lo += __popcll(__ballot(hit && i < x_lo));
                    below_hi += __popcll(__ballot(hit && i < x_hi));
                }
            }
            before[u] = b;
        }
        return wtot;
    };
    // ---- count this expert's pairs and publish the count
    int wave_all = 0, wtot = 0;
    for (int base0 = 0; base0 < a.P; base0 += kChunk) {
        if (base0 > 0) load_chunk(base0);
        wtot = count_chunk(base0, keep);
        wave_all += wtot;
    }
    if (lane == 0) { s_cnt[wave] = wave_all; s_below[0][wave] = below_lo; s_below[1][wave] = below_hi; }
    __syncthreads();
    int cnt = 0, lo_cnt = 0, hi_cnt = 0;
#pragma unroll
    for (int w = 0; w < kRouteWaves; ++w) { cnt += s_cnt[w]; lo_cnt += s_below[0][w]; hi_cnt += s_below[1][w]; }
    const int tiled = keep ? hi_cnt - lo_cnt : cnt;  // rows of this expert that get tiles
    if (tid == 0) {
        __hip_atomic_store(&counts[e], ((unsigned long long)tag << 32) | (unsigned)cnt, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
        if (keep)
            __hip_atomic_store(&kept[e], ((unsigned long long)tag << 32) | (unsigned)tiled, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
    }

    // ---- stable placement, chunk by chunk
    const bool in_lds = cnt <= kSegTokLds;
    int seg_lo = 0, first = 0;
    int running = 0;                                 // matches of the chunks before this one
    int par = 0;                                     // wave_tot is double-buffered over the chunks
    for (int base0 = 0; base0 < a.P || base0 == 0; base0 += kChunk, par ^= 1) {   // (once even without pairs)
        if (!one_chunk) {
            load_chunk(base0);
            wtot = count_chunk(base0, false);
        }
        if (lane == 0) wave_tot[par][wave] = wtot;
        __syncthreads();
        int wbase = 0, ctot = 0;
#pragma unroll
        for (int w = 0; w < kRouteWaves; ++w) {
            const int c = wave_tot[par][w];
            if (w < wave) wbase += c;
            ctot += c;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int lp = wbase + before[u];
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (vv[u][k] == e) cidx[lp++] = (unsigned short)(lane_off + u * 256 + k);
        }
        if (e == 0 && a.pair_pos) {
            // an id outside [0, E): the pair is nowhere in the sorted order
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int i = base0 + lane_off + u * 256 + k;
                    if (i < a.P && (unsigned)vv[u][k] >= (unsigned)a.E) a.pair_pos[i] = -1;
                }
        }
        if (base0 == 0 && wave == 0) {
            // the counts of the experts before e: segment offset and first tile index
            int off = 0, tiles = 0;
            bool gave_up = false;
            const long long t0 = wall_clock64();
            auto wait_for = [&](const unsigned long long* word) {
                for (;;) {
                    const unsigned long long v = __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if ((unsigned)(v >> 32) == tag) return (int)(unsigned)v;
                    if (wall_clock64() - t0 > a.wait_ticks) { gave_up = true; return 0; }
                    __builtin_amdgcn_s_sleep(1);
                }
            };
            for (int i = lane; i < e; i += 64) {
                const int c = wait_for(&counts[i]);
                const int r = keep ? wait_for(&kept[i]) : c;
                off += c;
                tiles += ((r + a.bm - 1) / a.bm) * a.tiles_n;
            }
            for (int sft = 32; sft > 0; sft >>= 1) {
                off += __shfl_down(off, sft);
                tiles += __shfl_down(tiles, sft);
            }
            if (gave_up) *a.err = 1;
            if (lane == 0) { s_seg_lo = off; s_first = tiles; }
        }
        __syncthreads();
        if (base0 == 0) { seg_lo = s_seg_lo; first = s_first; }
        for (int t = tid; t < ctot; t += kRouteThreads) {
            const int i = base0 + cidx[t], tk = i / a.topk, pos = seg_lo + running + t;
            a.sorted_token[pos] = tk;
            if (a.pair_pos) a.pair_pos[i] = pos;
            if (in_lds) seg_tok[running + t] = tk;
        }
        running += ctot;
    }
    const int seg_hi = seg_lo + cnt;
    if (tid == 0) {
        a.seg_off[e] = seg_lo;
        if (e == a.E - 1) {
            a.seg_off[a.E] = seg_hi;
            const int total = first + ((tiled + a.bm - 1) / a.bm) * a.tiles_n;
            *a.n_tiles_dev = total <= a.tab_capacity ? total : 0;   // the capacity is an upper bound by construction
            // every workgroup has taken its ticket and read the call word by now (their counts are all in)
            __hip_atomic_store(ticket_word, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(call_word, tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    // ---- tile entries (they read this expert's sorted tokens: from LDS, or, for a longer segment, from sorted_token
    // as this same workgroup wrote it above)
    __threadfence_block();
    __syncthreads();
    auto tok_at = [&](int pos) { return in_lds ? seg_tok[pos - seg_lo] : a.sorted_token[pos]; };
    const int row_lo = keep ? seg_lo + lo_cnt : seg_lo, row_hi = row_lo + tiled;
    const int mt = (tiled + a.bm - 1) / a.bm;
    if (first + mt * a.tiles_n > a.tab_capacity) return;
    for (int k = tid; k < mt * a.tiles_n; k += kRouteThreads) {
        const int n = k / mt, m = k - n * mt;
        MoeTile t;
        t.expert = e;
        t.m0 = row_lo + m * a.bm;
        t.m_end = min(t.m0 + a.bm, row_hi);
        t.n_tile = n;
        // tokens rise inside a segment: the first and last token bound the rows of T this tile reads
        const int tok_lo = tok_at(t.m0), tok_hi = tok_at(t.m_end - 1);
        t.f_lo = min(tok_lo / a.rows_per_flag, a.n_flags - 1);
        t.f_hi = min(tok_hi / a.rows_per_flag, a.n_flags - 1);
        t.st_lo = t.m0;
        t.st_hi = t.m_end;
        a.tile_tab[first + k] = t;
    }
}

// Top-k reduction (Section 4.1, "MoE ReduceScatter", the step between the grouped GEMM and the reduce scatter):
// every token's `topk` rows of Y are weighted with its gate values and summed in slot order, fp32, starting from the
// first product.  Streaming, one float4 column chunk per lane, tokens of this rank first (their slice is what the
// reducer waits for).  A lane works on U tokens at a time: the row of a pair is found through pair_pos, so every
// product is two loads in a row (index, then data); with U tokens in hand the U indices are in flight together and
// then the U rows, instead of one such chain after the other.
__global__ __launch_bounds__(256) void topk_reduce_kernel(const TopkReduceArgs a)
{
    typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
    constexpr int U = 4;
    const int n4 = a.N / 4;
    const int own_n = a.own_hi - a.own_lo;
    const int n_tok = a.Z_other ? a.T : own_n;                 // tokens that are reduced: own first, then the others
    const long long total = (long long)((n_tok + U - 1) / U) * n4;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
        const int grp = (int)(i / n4);
        const int j = (int)(i - (long long)grp * n4);
        int tk[U];
        f32x4 z[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int v = grp * U + u;                          // place in the order
            int t = -1;
            if (v < n_tok) {
                if (v < own_n) t = a.own_lo + v;
                else { t = v - own_n; if (t >= a.own_lo) t += own_n; }
            }
            tk[u] = t;
            z[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        for (int s = 0; s < a.topk; ++s) {
            int p[U];
            float g[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                p[u] = tk[u] >= 0 ? a.pair_pos[tk[u] * a.topk + s] : -1;
                g[u] = tk[u] >= 0 ? a.gate[tk[u] * a.topk + s] : 0.f;
            }
            f32x4 y[U];
#pragma unroll
            for (int u = 0; u < U; ++u)       // (a pair with an invalid expert id has no row: it contributes nothing)
                y[u] = p[u] >= 0 ? __builtin_nontemporal_load((const f32x4*)(a.Y + (long long)p[u] * a.N) + j) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (p[u] >= 0) z[u] = z[u] + g[u] * y[u];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = tk[u];
            if (t < 0) continue;
            const bool own = t >= a.own_lo && t < a.own_hi;
            f32x4* dst = own ? (f32x4*)(a.Z_own + (long long)(t - a.own_lo) * a.N) + j : (f32x4*)(a.Z_other + (long long)t * a.N) + j;
            *dst = z[u];
        }
    }
}

hipError_t launch_topk_reduce(const TopkReduceArgs& a, int n_workgroups, hipStream_t stream)
{
    hipLaunchKernelGGL(topk_reduce_kernel, dim3(n_workgroups), dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_moe_route(const MoeRouteArgs& a, hipStream_t stream)
{
    if (a.E > kMoeMaxExperts || !a.ctrl || !a.err) return hipErrorInvalidValue;
    hipLaunchKernelGGL(moe_route_kernel, dim3(a.E), dim3(kRouteThreads), 0, stream, a);
    return hipGetLastError();
}

}  // namespace agg

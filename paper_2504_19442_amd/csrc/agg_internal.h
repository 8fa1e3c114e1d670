// Internal declarations shared by the translation units of libagg.so (HIP path only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/agg.h"

namespace agg {

constexpr int kMaxWorld = 64;          // kernel-argument arrays are sized for this many ranks
constexpr int kSignalStride = AGG_SIGNAL_STRIDE;
constexpr int kMaxRsChunks = 16;       // row chunks per GEMM-RS slice (each with its own counter and signal)

// What one GEMM launch needs.  A is row-major [M][K] bf16 (optionally gathered through row_index),
// B is [N][K] bf16 (K contiguous), C row-major.
struct GemmParams {
    const uint16_t* A;
    const uint16_t* A_local;   // AllGather-GEMM: this rank's own shard where the caller keeps it (nullptr = read it from A)
    int local_lo, local_hi;    // its rows in A
    const uint16_t* B;
    void* C;              // every row whose slice has no destination of its own
    long long lda, ldb, ldc;
    int M, N, K;
    int c_is_f32;
    int c_vec_ok;         // C, the slice destinations and their leading dimensions allow 16-byte row-chunk stores
    // tile schedule (Section 3.7: rank-rotated order, local shard first)
    int tiles_m, tiles_n;
    int panel_m;          // m-tiles per panel (a panel = the tiles of one shard step)
    int group_n;          // n-tiles per L2 block inside a panel
    int m_tile_start;     // m-tile holding this rank's first row
    int order;            // AGG_ORDER_*: how the m-tiles are walked
    int tiles_per_shard, tiles_per_chunk, world, rank;   // for the sub-chunk order
    // signals (nullptr = un-gated)
    const int* flags;
    int epoch;
    const int* epoch_ptr;         // not null: the epoch is read from this device word when the kernel starts
    int rows_per_flag;    // rows of A covered by one signal
    int n_flags;
    long long wait_ticks; // bound of a wait, in wall-clock ticks
    int* err;             // device word: set to 1 when a wait is given up
    // GEMM-RS scatter (n_slices > 0): the rows are cut into slices of slice_rows; slice w is stored at
    // slice_dst[w] (row index relative to the slice, leading dimension ldc_slice) where that is not null, else in C.
    // Each slice is cut further into slice_chunks row chunks of chunk_rows.  Tiles touching chunk c of slice w count
    // up slice_ctr[w * slice_chunks + c]; the last one raises slice_flag[w][c * kSignalStride] (where not null).
    int n_slices, slice_rows, slice_chunks, chunk_rows;
    long long ldc_slice;
    int* slice_ctr;
    void* slice_dst[kMaxWorld];
    int* slice_flag[kMaxWorld];
    // grouped (MoE) GEMM only: rows of A are gathered through row_index, tiles come from a table built on the device
    const int* row_index;         // row p of the output reads row row_index[p] of A
    const struct MoeTile* tile_tab;
    const int* n_tiles_dev;       // number of table entries (device word)
    long long b_group_stride;     // elements between the B matrices of consecutive groups (experts)
    unsigned a_bytes;             // size of A in bytes (bound of the gather)
};

// One output tile of the grouped GEMM: rows [m0, m_end) of the sorted pair list (inside one expert's segment),
// columns of n-tile n_tile, waiting for signals f_lo..f_hi; of its rows, [st_lo, st_hi) are stored (the routing
// kernel lists all of them; an empty range = the tile is skipped).
struct MoeTile {
    int expert, m0, m_end, n_tile, f_lo, f_hi, st_lo, st_hi;
};

struct MoeRouteArgs {
    const int* topk_ids;          // [P] = [Ttok * topk]
    int P, topk, E;
    int* seg_off;                 // [E + 1] out
    int* sorted_token;            // [P] out
    int* pair_pos;                // [P] out or nullptr: place of flat pair (token * topk + slot) in the sorted order
    int keep_lo, keep_hi;         // keep_lo < keep_hi: only rows of tokens in [keep_lo, keep_hi) are stored by the GEMM
    // tile table
    int bm, tiles_n, rows_per_flag, n_flags;
    MoeTile* tile_tab;
    int tab_capacity;
    int* n_tiles_dev;
    unsigned char* ctrl;          // the routing's control block (kMoeCtrlBytes of device memory, all zero before its first use)
    long long wait_ticks;         // bound of the wait for the other experts' counts, in wall-clock ticks
    int* err;                     // device word: set to 1 when that wait is given up
};
// Control block of the MoE routing: the tile count (int, read by the grouped GEMM), the number of finished routing
// calls, the ticket counter, and two tagged counts per expert (its pairs; those of them that get tiles).
constexpr int kMoeMaxExperts = 4096;
constexpr size_t kMoeCtrlCall = 8, kMoeCtrlTicket = 16, kMoeCtrlCounts = 256;
constexpr size_t kMoeCtrlKept = kMoeCtrlCounts + (size_t)kMoeMaxExperts * 8;
constexpr size_t kMoeCtrlBytes = kMoeCtrlKept + (size_t)kMoeMaxExperts * 8;
hipError_t launch_moe_route(const MoeRouteArgs& a, hipStream_t stream);

// Top-k reduction of MoE + ReduceScatter: Z[t, :] = sum_s gate[t, s] * Y[pair_pos[t * topk + s], :]
struct TopkReduceArgs {
    const float* Y;               // [T * topk, N] fp32, rows in routing order
    const int* pair_pos;
    const float* gate;            // [T, topk]
    int T, topk, N;
    int own_lo, own_hi;           // tokens of this rank: their rows go to Z_own (row t - own_lo) ...
    float* Z_own;
    float* Z_other;               // ... all other tokens to row t of Z_other (nullptr: not computed)
};
hipError_t launch_topk_reduce(const TopkReduceArgs& a, int n_workgroups, hipStream_t stream);
hipError_t launch_gemm_grouped(const GemmParams& p, int cfg, int grid, hipStream_t stream);

// A tile configuration = a tile shape (bits 0-1) and the MFMA form of the main loop (bit 2): v_mfma_f32_32x32x16_bf16,
// or, with TILE_K32, v_mfma_f32_16x16x32_bf16 (half the accumulator traffic per flop: the chip holds a higher clock).
enum TileConfig { TILE_256x224 = 0, TILE_128x128 = 1, TILE_256x256 = 2, TILE_128x256 = 3, TILE_K32 = 4, TILE_CONFIGS = 8 };

struct TileShape { int bm, bn; };
inline TileShape tile_shape(int cfg)
{
    switch (cfg & 3) {
        case TILE_256x224: return {256, 224};
        case TILE_256x256: return {256, 256};
        case TILE_128x256: return {128, 256};
        default: return {128, 128};
    }
}

hipError_t launch_gemm(const GemmParams& p, int cfg, int grid, hipStream_t stream);

struct ProducerArgs {
    const void* src[kMaxWorld];   // src[j] = local buffer of the j-th shard to arrive
    int rank_of[kMaxWorld];       // its rank (destination slot in T)
    int n_jobs;
    char* T;
    long long shard_bytes;
    long long chunk_bytes;
    int chunks_per_shard;
    int* flags;
    int* counters;
    int epoch;
    const int* epoch_ptr;         // not null: the epoch is read from this device word when the kernel starts
    int team;                     // workgroups that share one chunk (set by launch_producer)
    int link_wgs;                 // full-mesh mode: workgroups per link (set by launch_producer_links)
    double ticks_per_byte;        // full-mesh mode: wall-clock ticks a link takes per byte (0 = not paced)
};
hipError_t launch_producer(const ProducerArgs& a, int n_workgroups, int threads, hipStream_t stream);
hipError_t launch_producer_links(const ProducerArgs& a, int n_workgroups, hipStream_t stream);
hipError_t launch_signal_set(int* flag, int value, const int* value_ptr, hipStream_t stream);
hipError_t launch_epoch_advance(int* epoch_word, hipStream_t stream);
hipError_t launch_signal_probe(const int* flag, int value, long long ticks, int* seen, hipStream_t stream);

hipError_t launch_transpose_kn(const uint16_t* B_kn, long long ldb, int K, int N, uint16_t* B_nk, hipStream_t stream);
hipError_t launch_mfma_ceiling(float* sink, int grid, int iters, int constant_operands, hipStream_t stream);

struct ReduceArgs {
    const float* slot[kMaxWorld];
    int W;
    long long n_vec4;             // number of float4 elements
    long long row_vec4;           // float4 per row (N / 4) when ldr != N, else 0
    void* R;
    long long ldr;
    int r_is_f32;
    int N;
    const int* flags;
    int flag_step;                // signal index of slot w = w * flag_step
    int chunks;                   // > 1: slot w arrives in this many row chunks, chunk c on signal w * flag_step + c
    long long chunk_vec4;         // float4 elements per chunk
    int epoch;
    const int* epoch_ptr;         // not null: the epoch is read from this device word when the kernel starts
    long long wait_ticks;
    int* err;
};
void tune_table_put(int W, int M, int N, int K, const agg_tune_result& r);   // the process-wide table of tuned configurations
hipError_t launch_reduce(const ReduceArgs& a, int n_workgroups, hipStream_t stream, bool beside_gemm);

}  // namespace agg

struct agg_ctx {
    int W, rank;
    size_t shard_bytes;
    int n_signals;
    int epoch;
    uint64_t wait_limit_us;
    long long wall_khz;
    int num_cus;
    char* staging;       // T
    int* signals;        // S, n_signals * stride
    int* counters;       // per-signal arrival counters (producer), + GEMM-RS tile counter
    int* err;            // time-out record
    int* epoch_word;     // device copy of the epoch (source of the SDMA signal copies; the epoch itself in device-epoch mode)
    int device_epoch;    // 1: launches read the epoch from epoch_word when they start (HIP graph replay)
    int device;
    int tile_config;     // -1 = automatic
    int tile_order;      // AGG_ORDER_*
    int rs_own_last;     // gemm_rs computes the own slice last (1) or first (0)
    int rs_chunks;       // row chunks per GEMM-RS slice and reducer slot, each with a signal of its own (>= 1)
    int producer_wgs;    // workgroups of the producer kernel when the caller passes 0 (0 = one per CU)
    const void* local_shard;  // see agg_set_local_shard
    double link_GBps;    // pace of a link of the full-mesh producer (0 = not paced)
    hipStream_t producer_stream, consumer_stream;
    // grouped GEMM workspace (sized by agg_reserve_moe; no other call allocates it)
    int* moe_ws;          // the MoE routing's control block (kMoeCtrlBytes; its first word is the tile count of the launch under way)
    agg::MoeTile* moe_tab;
    int moe_tab_cap;
    uint16_t* b_nk;       // [N][K] copy of a B that was given as [K][N] (sized by agg_reserve_b_kn)
    size_t b_nk_elems;
    hipEvent_t b_nk_free;     // recorded behind the last GEMM that read b_nk, on b_nk_stream
    hipStream_t b_nk_stream;
    int b_nk_in_use;
    unsigned char* static_scratch;   // device address of the library's static scratch array on this context's GPU
    int can_wait_value;  // the device supports stream waits on a memory word
    hipEvent_t gemm_done; // GEMM-RS: orders the reducer after the GEMM where it does not
};

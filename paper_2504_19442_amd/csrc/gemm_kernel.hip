// Signal-gated bf16 GEMM for gfx950: the AllGather-GEMM consumer (Section 2.3, Figure 4) and the
// un-gated producer GEMM of GEMM+ReduceScatter (Section 3.3).
//
// One persistent workgroup of 4 waves per CU walks a list of BM x BN output tiles.  The tile order is
// the rank-rotated one of Section 3.7 (the panel holding the local shard first, then the shards in the
// order they are pulled), cut into blocks of 32 tiles that share A rows and B columns so that the 32
// workgroups of one XCD, which share an L2, work on neighbouring tiles.  Before a tile's first load of A
// the workgroup waits (acquire) for the signals covering the tile's rows -- the wait / consume_token
// pair of Section 2.2.
//
// Main loop: K is cut into steps of 32.  A and B tiles go from global memory straight into LDS
// (global_load_lds_dwordx4, 16 bytes per lane) through a ring of NS stages, so NS-1 steps of loads are
// in flight while one is computed.  Rows are 64 bytes in LDS; the 16-byte chunk c of row r sits in slot
// c ^ ((r >> 2) & 3), which makes the ds_read_b128 operand fetches bank-conflict free.  Each wave owns
// BM/4 rows and all BN columns of the tile and feeds v_mfma_f32_32x32x16_bf16 from two register sets
// of fragments that are refilled one half-step ahead of their use.  One workgroup barrier per step.
#include "agg_internal.h"

namespace agg {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

// s_waitcnt immediate that waits only for vmcnt <= n (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt_hi[15:14]).
__host__ __device__ constexpr int vmcnt_imm(int n) { return (n & 0xF) | (0x7 << 4) | (0xF << 8) | ((n >> 4) << 14); }

constexpr int BK = 32;                 // bf16 per K-step
constexpr int ROW_BYTES = BK * 2;      // 64-byte rows in LDS
constexpr int UNIT_ROWS = 16;          // one wave-wide 16-byte-per-lane load covers 16 rows

template <int BM, int BN, int NS>
struct Cfg {
    static constexpr int TM = BM / 4;            // rows per wave
    static constexpr int MB = TM / 32;           // 32x32 blocks per wave, M direction
    static constexpr int NB = BN / 32;           // and N direction
    static constexpr int A_UNITS = BM / UNIT_ROWS;
    static constexpr int B_UNITS = BN / UNIT_ROWS;
    static constexpr int UNITS = A_UNITS + B_UNITS;
    static constexpr int FULL = UNITS / 4;       // whole units per wave per stage
    static constexpr int REM = UNITS % 4;        // 0, or 2 (each of the two left-over units is loaded by a pair of waves: same data twice)
    static constexpr int L = FULL + (REM ? 1 : 0);   // load instructions per wave per stage
    static constexpr int STAGE_BYTES = (BM + BN) * ROW_BYTES;
    static constexpr int LDS_BYTES = STAGE_BYTES * NS;
    static_assert(BM % 128 == 0 && BN % 32 == 0, "tile shape");
    static_assert(A_UNITS % 4 == 0, "A units must split evenly over 4 waves");
    static_assert(REM == 0 || REM == 2, "unsupported unit count");
    static_assert(NS >= 3 && NS % 2 == 0, "ring needs at least 3 stages, and an even count for the fragment-set rotation");
    static_assert((NS - 2) * L <= 63, "vmcnt range");
};

template <int BM, int BN, int NS>
__global__ __launch_bounds__(256) void gemm_kernel(const GemmParams p)
{
    using C_ = Cfg<BM, BN, NS>;
    constexpr int MB = C_::MB, NB = C_::NB, L = C_::L, FULL = C_::FULL, TM = C_::TM;
    constexpr int H = NB / 2;            // column blocks of half-step 0 issued before the barrier
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- per-lane constants
    // global->LDS: lane l of a unit fills row l/4, slot l%4; the slot holds chunk (l%4) ^ ((row>>2)&3)
    const int ld_row = lane >> 2;
    const int ld_chunk = (lane & 3) ^ ((lane >> 4) & 3);
    // LDS->VGPR fragments: lane l reads row l%32, chunk 2*s + l/32, stored in slot chunk ^ ((row>>2)&3)
    int fr_off[2];
#pragma unroll
    for (int s = 0; s < 2; ++s)
        fr_off[s] = (lane & 31) * ROW_BYTES + (((2 * s + (lane >> 5)) ^ ((lane >> 2) & 3)) << 4);

    const int KT = p.K / BK;
    const int total_tiles = p.tiles_m * p.tiles_n;
    const int G = gridDim.x;
    const int g = blockIdx.x;
    const int xcd_slots = G >> 3;        // workgroups per XCD when G % 8 == 0

    for (int base = 0; base < total_tiles; base += G) {
        // ---- which tile: consecutive tiles of the list go to the workgroups of one XCD
        int t;
        if ((G & 7) == 0) t = base + (g & 7) * xcd_slots + (g >> 3); else t = base + g;
        if (t >= total_tiles) continue;
        int m_tile, n_tile;
        {
            const int per_panel = p.panel_m * p.tiles_n;
            const int panel = t / per_panel;
            const int pm = min(p.panel_m, p.tiles_m - panel * p.panel_m);
            const int q = t - panel * per_panel;
            const int blk = q / (pm * p.group_n);
            const int r = q - blk * pm * p.group_n;
            const int gn = min(p.group_n, p.tiles_n - blk * p.group_n);
            const int mi = r / gn;
            n_tile = blk * p.group_n + (r - mi * gn);
            m_tile = (p.m_tile_start + panel * p.panel_m + mi) % p.tiles_m;
        }
        const int m0 = m_tile * BM, n0 = n_tile * BN;

        // ---- wait for the signals covering rows [m0, min(m0+BM, M))  (wait + consume_token, Section 2.2)
        if (p.flags) {
            const int f_lo = m0 / p.rows_per_flag;
            const int f_hi = min((min(m0 + BM, p.M) - 1) / p.rows_per_flag, p.n_flags - 1);
            int gave_up = 0;
            for (int f = f_lo + tid; f <= f_hi; f += 256) {
                const int* fp = p.flags + (long long)f * kSignalStride;
                const long long t0 = wall_clock64();
                while (__hip_atomic_load(fp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < p.epoch) {
                    if (__hip_atomic_load(p.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0 ||
                        wall_clock64() - t0 > p.wait_ticks) {
                        gave_up = 1;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(1);
                }
            }
            if (gave_up) __hip_atomic_store(p.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            if (__syncthreads_or(gave_up)) return;   // the launch drains; agg_status reports the time-out
        }

        // ---- per-tile load offsets (bytes from the tile's A / B origin; rows past the edge are clamped)
        const unsigned char* a_base = (const unsigned char*)(p.A + (long long)m0 * p.lda);
        const unsigned char* b_base = (const unsigned char*)(p.B + (long long)n0 * p.ldb);
        const int m_last = p.M - 1 - m0, n_last = p.N - 1 - n0;
        unsigned ld_off[L];
#pragma unroll
        for (int i = 0; i < L; ++i) {
            const int u = (i < FULL) ? wave + 4 * i : 4 * FULL + (wave >> 1);
            if (u < C_::A_UNITS) {
                const int r = min(u * UNIT_ROWS + ld_row, m_last);
                ld_off[i] = (unsigned)(r * (int)p.lda * 2 + ld_chunk * 16);
            } else {
                const int r = min((u - C_::A_UNITS) * UNIT_ROWS + ld_row, n_last);
                ld_off[i] = (unsigned)(r * (int)p.ldb * 2 + ld_chunk * 16);
            }
        }

        auto load_stage = [&](int st, int kt) {
            const unsigned char* ak = a_base + (long long)kt * ROW_BYTES;
            const unsigned char* bk = b_base + (long long)kt * ROW_BYTES;
#pragma unroll
            for (int i = 0; i < L; ++i) {
                const int u = (i < FULL) ? wave + 4 * i : 4 * FULL + (wave >> 1);
                // whether unit i of this wave is an A or a B unit is the same for all four waves
                const bool is_a = ((i < FULL) ? 4 * i : 4 * FULL) < C_::A_UNITS;
                const unsigned char* src = (is_a ? ak : bk) + ld_off[i];
                unsigned char* dst = lds + st * C_::STAGE_BYTES + u * 1024;
                __builtin_amdgcn_global_load_lds(GLOBAL_PTR(src), LDS_PTR(dst), 16, 0, 0);
            }
        };

        // four fragment sets: set 2*(kt&1) + s holds half-step s of step kt, so a set is refilled a whole
        // half-step before it is used and never while MFMAs that read it are still to be issued
        bf16x8 fa[4][MB], fb[4][NB];
        auto read_frags = [&](int st, int s, int set) {
            const unsigned char* sa = lds + st * C_::STAGE_BYTES + wave * TM * ROW_BYTES + fr_off[s];
            const unsigned char* sb = lds + st * C_::STAGE_BYTES + BM * ROW_BYTES + fr_off[s];
#pragma unroll
            for (int i = 0; i < MB; ++i) fa[set][i] = *(const bf16x8*)(sa + i * 32 * ROW_BYTES);
#pragma unroll
            for (int j = 0; j < NB; ++j) fb[set][j] = *(const bf16x8*)(sb + j * 32 * ROW_BYTES);
        };

        f32x16 acc[MB][NB];
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

        auto mma = [&](int set, int j_lo, int j_hi) {
#pragma unroll
            for (int j = j_lo; j < j_hi; ++j)
#pragma unroll
                for (int i = 0; i < MB; ++i)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][i], fb[set][j], acc[i][j], 0, 0, 0);
        };

        // ---- prologue: NS-1 stages in flight (steps past the end re-load the last step: harmless, and it
        // keeps the number of outstanding loads per wave the same on every path)
#pragma unroll
        for (int i = 0; i < NS - 1; ++i) load_stage(i, min(i, KT - 1));
        __builtin_amdgcn_s_waitcnt(vmcnt_imm((NS - 2) * L));
        __builtin_amdgcn_s_barrier();
        read_frags(0, 0, 0);

        // ---- main loop, unrolled over the ring so that stage and set indices are constants; the only
        // branches are the loop exits, so the body stays one straight line for the scheduler
        for (int kt0 = 0;; kt0 += NS) {
#pragma unroll
            for (int st = 0; st < NS; ++st) {
                const int kt = kt0 + st;
                const int cur = 2 * (st & 1), nxt = 2 * ((st + 1) & 1);
                // (A) first part of half-step 0 on the matrix pipe while the fragments of half-step 1 leave LDS
                mma(cur, 0, H);
                read_frags(st, 1, cur + 1);
#pragma unroll
                for (int q = 0; q < MB * H; ++q) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
                    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);   // two LDS reads
                }
                __builtin_amdgcn_sched_barrier(0);
                // stage kt+1 has landed for this wave once at most the younger stages are outstanding
                __builtin_amdgcn_s_waitcnt(vmcnt_imm((NS - 3) * L));
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
                // (B) every wave is past its reads of stage kt-1: refill it with step kt+NS-1, fetch the next
                // step's first fragments (early, so they are back before part C ends), rest of half-step 0
                mma(cur, H, NB);
                read_frags((st + 1) % NS, 0, nxt);
                load_stage((st + NS - 1) % NS, min(kt + NS - 1, KT - 1));
#pragma unroll
                for (int q = 0; q < MB * (NB - H); ++q) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
                    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);   // two LDS reads
                    __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);   // address arithmetic
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // one global->LDS load
                }
                __builtin_amdgcn_sched_barrier(0);
                // (C) half-step 1
                mma(cur + 1, 0, NB);
                __builtin_amdgcn_sched_barrier(0);
                if (kt + 1 >= KT) goto k_done;
            }
        }
    k_done:

        // ---- epilogue: accumulators to C.  32x32 block layout: lane l holds column l%32 and, in
        // register v, row 8*(v/4) + 4*(l/32) + v%4.
        {
            const int col = n0 + (lane & 31);
            const int row_w = m0 + wave * TM + 4 * (lane >> 5);
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = row_w + i * 32 + 8 * (v >> 2) + (v & 3);
                    if (row < p.M) {
                        void* cbase = p.C;
                        long long ldc = p.ldc;
                        long long rr = row;
                        if (p.C_own && row >= p.own_lo && row < p.own_hi) {
                            cbase = p.C_own;
                            ldc = p.ldc_own;
                            rr = row - p.own_lo;
                        }
                        if (cbase) {
#pragma unroll
                            for (int j = 0; j < NB; ++j) {
                                const int c = col + j * 32;
                                if (c < p.N) {
                                    if (p.c_is_f32)
                                        ((float*)cbase)[rr * ldc + c] = acc[i][j][v];
                                    else
                                        ((__bf16*)cbase)[rr * ldc + c] = (__bf16)acc[i][j][v];
                                }
                            }
                        }
                    }
                }
        }

        // GEMM-RS: count finished tiles of the own slice; the last one raises the producer signal
        if (p.done_ctr && m0 < p.own_hi && m0 + BM > p.own_lo) {
            __syncthreads();     // all stores of this tile issued
            if (tid == 0) {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
                const int prev = __hip_atomic_fetch_add(p.done_ctr, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
                if (prev == p.done_target - 1) {
                    __hip_atomic_store(p.done_ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(p.done_flag, p.epoch, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }

        // the ring is reused by the next tile: drain this tile's last (redundant) loads and reads first
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        __syncthreads();
    }
}

template <int BM, int BN, int NS>
static hipError_t launch_cfg(const GemmParams& p, int grid, hipStream_t stream)
{
    using C_ = Cfg<BM, BN, NS>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)gemm_kernel<BM, BN, NS>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C_::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((gemm_kernel<BM, BN, NS>), dim3(grid), dim3(256), C_::LDS_BYTES, stream, p);
    return hipGetLastError();
}

hipError_t launch_gemm(const GemmParams& p, int cfg, int grid, hipStream_t stream)
{
    switch (cfg) {
        case TILE_256x224: return launch_cfg<256, 224, 4>(p, grid, stream);
        case TILE_256x256: return launch_cfg<256, 256, 4>(p, grid, stream);
        default: return launch_cfg<128, 128, 4>(p, grid, stream);
    }
}

}  // namespace agg

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
// Main loop: K is cut into stages of 64, so that every row of a tile is fetched as one whole 128-byte line
// (the L2 hands out lines: asking for half a line at a time halves its useful bandwidth).  A and B tiles go
// from global memory straight into LDS (buffer_load_dwordx4 ... lds, 16 bytes per lane) into a ring that takes
// up nearly all of the LDS (two stages and a third of a third one).  Rows are 128 bytes in LDS; the 16-byte
// chunk c of row r sits in slot c ^ ((r >> 1) & 7), which makes the ds_read_b128 operand fetches bank-conflict
// free.  Each wave owns BM/4 rows and all BN columns of the tile.  Two forms of the loop (template parameter MF):
//   MF = 16: v_mfma_f32_16x16x32_bf16.  A stage is two half-steps of K = 32; a half-step is BN/16 groups of MFMAs, group j
//            using the B fragment of column block j against the wave's A fragments; the B fragment registers
//            are refilled for the next half-step as soon as their group is done.  Half the accumulator traffic per
//            flop of the other form: the chip, which is power-limited under this load, holds a higher clock.
//   MF = 32: v_mfma_f32_32x32x16_bf16.  A stage is four quarter-steps of K = 16, fragments double-buffered.
// One workgroup barrier per stage; memory instructions are dealt out between the MFMAs (a wave issues in
// order, and bunches of memory instructions between two MFMAs starve the matrix pipe).
// The MFMA computes the transposed block (B fragment as first operand), so that a lane ends up holding
// four consecutive columns of one output row; the epilogue stages each wave's rows through LDS and
// stores them to C as whole 16-byte row chunks.
//
// Registers: the fp32 accumulators live in accumulator registers a0..a(ACC-1) that only the inline
// asm of this file touches (MFMA, zeroing, read-out); the compiler allocates the ordinary registers and is
// capped so that the kernel takes at most 448 of the 512 registers of a SIMD.  The rest is what lets one
// wave of a small kernel (the producer's copy waves, the reducer) run beside a consumer wave on every
// SIMD: communication and computation share all CUs instead of splitting them (Section 3.8).
#pragma once
#include "agg_internal.h"

#if defined(__HIP_DEVICE_COMPILE__) && !defined(__gfx950__)
#error "this kernel names gfx950 instructions and registers (MFMA forms, accumulator registers, global->LDS loads)"
#endif

#include <numeric>
#include <type_traits>
#include <utility>

namespace agg {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;

#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
typedef __attribute__((address_space(3))) unsigned char lds_byte;
typedef __attribute__((address_space(3))) const bf16x8 lds_frag;

// Raw buffer descriptor over `bytes` bytes at p: loads whose per-lane offset is >= bytes return zero, which
// is how rows past the edge of A or B are masked.  0x00020000 = 32-bit data format, no swizzle (gfx9 family).
__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}

// s_waitcnt immediate that waits only for vmcnt <= n (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt_hi[15:14]).
__host__ __device__ constexpr int vmcnt_imm(int n) { return (n & 0xF) | (0x7 << 4) | (0xF << 8) | ((n >> 4) << 14); }

// compile-time loop: f(std::integral_constant<int, I>) for I in [0, N)
template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// ---- accumulator registers, touched only here.  Block b is a[16b : 16b+15].
template <int BLK>
__device__ __forceinline__ void mfma_acc(const bf16x8& a, const bf16x8& b)
{
    asm volatile("v_mfma_f32_32x32x16_bf16 a[%2:%3], %0, %1, a[%2:%3]" ::"v"(a), "v"(b), "n"(BLK * 16), "n"(BLK * 16 + 15));
}
// the 16x16x32 form: block b is a[4b : 4b+3]
template <int BLK>
__device__ __forceinline__ void mfma_acc16(const bf16x8& a, const bf16x8& b)
{
    asm volatile("v_mfma_f32_16x16x32_bf16 a[%2:%3], %0, %1, a[%2:%3]" ::"v"(a), "v"(b), "n"(BLK * 4), "n"(BLK * 4 + 3));
}
template <int R>
__device__ __forceinline__ void acc_zero()
{
    asm volatile("v_accvgpr_write_b32 a[%0], 0" ::"n"(R));
}
template <int R>
__device__ __forceinline__ float acc_read()
{
    float x;
    asm volatile("v_accvgpr_read_b32 %0, a[%1]" : "=v"(x) : "n"(R));
    return x;
}

constexpr int BK = 64;                 // bf16 per stage
constexpr int ROW_BYTES = BK * 2;      // 128-byte rows in LDS: one cache line per row and stage
constexpr int UNIT_ROWS = 8;           // one wave-wide 16-byte-per-lane load covers 8 rows
[[maybe_unused]] constexpr int QS = 4;   // quarter-steps (K = 16 each) per stage

template <int BM, int BN>
struct Cfg {
    static constexpr int TM = BM / 4;            // rows per wave
    static constexpr int MB = TM / 32;           // 32x32 blocks per wave, M direction
    static constexpr int NB = BN / 32;           // and N direction
    static constexpr int ACC = MB * NB * 16;     // accumulator registers per lane
    static constexpr int A_UNITS = BM / UNIT_ROWS;
    static constexpr int B_UNITS = BN / UNIT_ROWS;
    static constexpr int UNITS = A_UNITS + B_UNITS;
    static constexpr int L = UNITS / 4;          // load instructions per wave per stage
    static constexpr int STAGE_BYTES = (BM + BN) * ROW_BYTES;
    // The LDS ring holds RW loads per wave (4 KiB each: the same load of all four waves), a stage is L of them.
    // RW >= 2 L; RW need not be a multiple of L: the stream of loads simply wraps around the ring, so that the
    // whole LDS is used as look-ahead even when only 2 1/3 stages fit.
    static constexpr int RW = (BN == 256) ? 36 : (BM == 256) ? 35 : 32;
    static constexpr int RING_BYTES = RW * 4096;
    static constexpr int PERIOD = std::lcm(L, RW) / L;     // stages after which ring positions repeat
    // epilogue staging: each wave stages 32 rows x BN columns at a time
    static constexpr int PITCH_BF16 = BN * 2 + 16;
    static constexpr int PITCH_F32 = BN * 4 + 16;
    static constexpr int LDS_BYTES = (RING_BYTES > 4 * 32 * PITCH_F32) ? RING_BYTES : 4 * 32 * PITCH_F32;
    static_assert(BM % 128 == 0 && BN % 32 == 0, "tile shape");
    static_assert(A_UNITS % 4 == 0 && B_UNITS % 4 == 0, "units must split evenly over 4 waves");
    static_assert(RW >= 2 * L && RW <= 63, "ring: at least two stages, and the prologue's loads fit the vmcnt range");
    static_assert(PERIOD <= 9, "the main loop is unrolled over PERIOD stages");
    static_assert(ACC == 64 || ACC == 128 || ACC == 224 || ACC == 256, "add a reservation line for this accumulator count");
    // One quarter-step is SLOTS = MB*NB MFMAs.  Its memory instructions, in order: LQ global->LDS loads
    // (while a stage's loads are being issued: the three quarter-steps after a barrier), then the F = MB+NB
    // fragment reads of the next quarter-step.  They are dealt out QUOTA per MFMA slot.
    static constexpr int SLOTS = MB * NB;
    static constexpr int F = MB + NB;
    static constexpr int LQ = (L + 2) / 3;   // loads per quarter-step while a batch is issued
    static constexpr int QUOTA = (LQ + F + SLOTS - 1) / SLOTS;

    // ---- the 16x16x32 form of the main loop (MF = 16).  A stage is two half-steps of K = 32; a half-step is NB16 groups
    // of MB16 MFMAs, group j working on the B fragment of column block j and all MB16 A fragments of the wave.
    static constexpr int MB16 = TM / 16;
    static constexpr int NB16 = BN / 16;
    static constexpr int DLY = 3;                // the stage's barrier sits after group DLY - 1 of the second half-step
    static constexpr int NS = NB16 * MB16;       // MFMA slots per half-step: slot s = group s / MB16, row block s % MB16
    static constexpr int SB = DLY * MB16 - 1;    // the barrier follows the MFMA of this slot (second half-step)
    // The L loads that a barrier releases are issued one every PACE slots from the barrier on, through the rest of that
    // half-step and the next stage's first half-step: evenly, because the four waves share one path into LDS (a load
    // of one wave occupies it for 16 cycles, one MFMA slot) and bunched loads make the waves queue up at issue.
    static constexpr int PACE = (2 * NS - SB - 1) / L > 0 ? (2 * NS - SB - 1) / L : 1;
    static constexpr int LH1_ = (NS - SB + PACE - 1) / PACE;
    static constexpr int LH1 = LH1_ < L ? LH1_ : L;   // loads issued in the rest of the second half-step
    static constexpr int LH0 = L - LH1;          // the others: in the next stage's first half-step
    static constexpr int P0 = RW - L + LH1;      // loads issued by the prologue
    static_assert(SB + (L - 1) * PACE < 2 * NS && P0 >= L && P0 <= 63, "load schedule of the 16x16x32 loop");
    static_assert(DLY + MB16 <= NB16, "the reads of the next A fragments fit between the barrier and the end of the half-step");
    struct Op { int type, idx; };                // 0 none, 1 read B fragment idx, 2 read A fragment idx, 3 global->LDS load idx
    static constexpr int PER_SLOT = 3;
    struct Slots { Op op[NS][PER_SLOT]; bool complete; };
    // The memory operations of half-step h, placed behind the MFMA slots.  Each has an earliest slot: the refill of B
    // register set j after the last MFMA of group j (and, in the second half-step, not before the barrier); the reads
    // of the next A fragments one per group from group DLY on; the global->LDS loads one every PACE slots, from the barrier on.  They are
    // taken in that order, one per slot, two when three or more are ready; the last slot takes whatever is left.
    static constexpr Slots make_slots(int h)
    {
        Op ops[64] = {};
        int early[64] = {};
        int n = 0;
        for (int j = 0; j < NB16; ++j) {
            int e = j * MB16 + MB16 - 1;
            if (h == 1 && e < SB) e = SB;
            ops[n] = Op{1, j}; early[n++] = e;
        }
        for (int ia = 0; ia < MB16; ++ia) { ops[n] = Op{2, ia}; early[n++] = (DLY + ia) * MB16; }
        if (h == 1) for (int jj = 0; jj < LH1; ++jj) { ops[n] = Op{3, jj}; early[n++] = SB + jj * PACE; }
        else for (int jj = LH1; jj < L; ++jj) { ops[n] = Op{3, jj}; early[n++] = SB + jj * PACE - NS; }
        for (int a = 1; a < n; ++a)                      // stable insertion sort by earliest slot
            for (int b = a; b > 0 && early[b - 1] > early[b]; --b) {
                const Op to = ops[b]; ops[b] = ops[b - 1]; ops[b - 1] = to;
                const int te = early[b]; early[b] = early[b - 1]; early[b - 1] = te;
            }
        Slots S{};
        int next = 0;
        for (int s = 0; s < NS; ++s) {
            int ready = 0;
            for (int k = next; k < n && early[k] <= s; ++k) ++ready;
            int take = ready >= 3 ? 2 : (ready >= 1 ? 1 : 0);
            if (s == NS - 1) take = ready < PER_SLOT ? ready : PER_SLOT;
            for (int k = 0; k < take; ++k) S.op[s][k] = ops[next++];
        }
        S.complete = next == n;
        return S;
    }
    static_assert(make_slots(0).complete && make_slots(1).complete, "every memory operation of a half-step has a slot");
};

// Register budget: 448 of the 512 registers a SIMD has (see the file comment).
// GROUPED = the MoE grouped GEMM (Section 4.1): tiles come from a table built on the device, rows of A are gathered
// through row_index, B is the tile's expert's matrix, and rows at or past the tile's segment end are neither loaded
// (they read as zero) nor stored.
template <int BM, int BN, bool GROUPED, int MF>
__global__ __launch_bounds__(256) __attribute__((amdgpu_num_vgpr(192))) void gemm_kernel(const GemmParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)    // the body names gfx950 registers; the host pass only needs the launch stub
    using C_ = Cfg<BM, BN>;
    constexpr int MB = C_::MB, NB = C_::NB, L = C_::L, TM = C_::TM;
    // naming the last accumulator register makes the compiler reserve a0..a(ACC-1) for this kernel
    if constexpr (C_::ACC == 256) asm volatile("; accumulators a0..a255" ::: "a255");
    else if constexpr (C_::ACC == 224) asm volatile("; accumulators a0..a223" ::: "a223");
    else if constexpr (C_::ACC == 128) asm volatile("; accumulators a0..a127" ::: "a127");
    else asm volatile("; accumulators a0..a63" ::: "a63");
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- per-lane constants
    // global->LDS: lane l of a unit fills row l/8, slot l%8 of the unit's 8 rows; slot s of row r holds chunk
    // s ^ ((r >> 1) & 7).  With r = 8u + l/8 that is s ^ ((4u + l/16) & 7): two cases, u even and u odd.
    const int ld_row = lane >> 3;
    const int ld_chunk_even = (lane & 7) ^ ((lane >> 4) & 7);
    const int ld_chunk_odd = (lane & 7) ^ ((4 + (lane >> 4)) & 7);
    // LDS->VGPR fragments of quarter-step h: lane l reads row l%32, chunk 2h + l/32, from slot chunk ^ ((row>>1)&7)
    // (MF = 16: fragments are 16 rows x K = 32; in half-step h lane l reads row l%16, chunk 4h + l/16)
    int fr_off[MF == 16 ? 2 : QS];
    if constexpr (MF == 16) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
            fr_off[h] = (lane & 15) * ROW_BYTES + (((4 * h + (lane >> 4)) ^ ((lane >> 1) & 7)) << 4);
    } else {
#pragma unroll
        for (int h = 0; h < QS; ++h)
            fr_off[h] = (lane & 31) * ROW_BYTES + (((2 * h + (lane >> 5)) ^ ((lane >> 1) & 7)) << 4);
    }

    // LDS addresses as numbers: of the ring's start, and of this wave's quarter of ring position 0
    const unsigned lds_u = (unsigned)(unsigned long)(lds_byte*)LDS_PTR(lds);
    unsigned lds_wave = lds_u + wave * 1024;
    // MF = 16: a B fragment read is base + immediate; the immediate holds 16 bits, the ring is larger, so there are
    // three bases per half-step (ring offsets 0, 64 KiB, 128 KiB), refreshed once per stage so that they stay registers
    unsigned frb[2][3];
    if constexpr (MF == 16) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int k = 0; k < 3; ++k) frb[h][k] = lds_u + fr_off[h] + k * 65536;
    }

    const int KS = p.K / BK;             // stages
    // the epoch the signals are compared with: the host's value at launch, or (for launches recorded in a HIP graph)
    // the context's device word as it stands when the kernel starts
    const int epoch = p.epoch_ptr ? __hip_atomic_load(p.epoch_ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : p.epoch;
    const int total_tiles = GROUPED ? *p.n_tiles_dev : p.tiles_m * p.tiles_n;
    const int G = gridDim.x;
    const int g = blockIdx.x;
    const int xcd_slots = G >> 3;        // workgroups per XCD when G % 8 == 0

    for (int base = 0; base < total_tiles; base += G) {
        // ---- which tile: consecutive tiles of the list go to the workgroups of one XCD
        int t;
        if ((G & 7) == 0) t = base + (g & 7) * xcd_slots + (g >> 3); else t = base + g;
        if (t >= total_tiles) continue;
        int m0, n0, m_lim, f_lo = 0, f_hi = -1, expert = 0;
        int st_lo = 0, st_hi;                 // rows of the output that are stored: [st_lo, st_hi)
        bool from_local = false;
        if constexpr (GROUPED) {
            const MoeTile mt = p.tile_tab[t];
            expert = __builtin_amdgcn_readfirstlane(mt.expert);
            m0 = __builtin_amdgcn_readfirstlane(mt.m0);
            m_lim = __builtin_amdgcn_readfirstlane(mt.m_end);
            st_lo = __builtin_amdgcn_readfirstlane(mt.st_lo);
            st_hi = __builtin_amdgcn_readfirstlane(mt.st_hi);
            if (st_hi <= st_lo) continue;     // no row of this tile is wanted (MoE + ReduceScatter without Z_other)
            n0 = __builtin_amdgcn_readfirstlane(mt.n_tile) * BN;
            f_lo = __builtin_amdgcn_readfirstlane(mt.f_lo);
            f_hi = __builtin_amdgcn_readfirstlane(mt.f_hi);
        } else {
            int m_tile, n_tile;
            const int per_panel = p.panel_m * p.tiles_n;
            const int panel = t / per_panel;
            const int pm = min(p.panel_m, p.tiles_m - panel * p.panel_m);
            const int q = t - panel * per_panel;
            const int blk = q / (pm * p.group_n);
            const int r = q - blk * pm * p.group_n;
            const int gn = min(p.group_n, p.tiles_n - blk * p.group_n);
            const int mi = r / gn;
            n_tile = blk * p.group_n + (r - mi * gn);
            const int v = panel * p.panel_m + mi;            // place in the order of m-tiles
            if (p.order == AGG_ORDER_SUBCHUNK) {
                // the local shard, then sub-chunk 0 of every peer (in pull order), sub-chunk 1 of every peer, ...
                if (v < p.tiles_per_shard) {
                    m_tile = p.rank * p.tiles_per_shard + v;
                } else {
                    const int v2 = v - p.tiles_per_shard;
                    const int per_c = (p.world - 1) * p.tiles_per_chunk;
                    const int c = v2 / per_c, rem = v2 - c * per_c;
                    const int jj = rem / p.tiles_per_chunk, k = rem - jj * p.tiles_per_chunk;
                    const int shard = (p.rank + 1 + jj) % p.world;
                    m_tile = shard * p.tiles_per_shard + c * p.tiles_per_chunk + k;
                }
            } else {
                m_tile = (p.m_tile_start + v) % p.tiles_m;
            }
            m0 = m_tile * BM;
            n0 = n_tile * BN;
            m_lim = p.M;
            st_hi = p.M;
            // a tile that lies inside this rank's own shard reads it where the caller keeps it: nothing to wait for
            from_local = p.A_local && m0 >= p.local_lo && m0 + BM <= p.local_hi;
            if (p.flags && !from_local) {
                f_lo = m0 / p.rows_per_flag;
                f_hi = min((min(m0 + BM, p.M) - 1) / p.rows_per_flag, p.n_flags - 1);
            }
        }

        // ---- wait for the signals covering rows [m0, min(m0+BM, M))  (wait + consume_token, Section 2.2)
        if (p.flags && f_hi >= f_lo) {
            // Wave 0 polls (lane l takes signals f_lo + l, f_lo + l + 64, ...) and, once it has seen them all, executes
            // the acquire: the wave that observed the signals is the wave that orders the loads of A after them.  The
            // acquire invalidates this CU's L1 and this XCD's L2 lines of remotely written memory, so that no load of
            // A below is served from a line cached before the data arrived; one wave does it for the workgroup
            // (invalidates from all waves of all CUs queue up behind each other at the L2), and the barrier holds the
            // other waves back until it is done.
            int gave_up = 0;
            if (wave == 0) {
                for (int f = f_lo + lane; f <= f_hi; f += 64) {
                    const int* fp = p.flags + (long long)f * kSignalStride;
                    const long long t0 = wall_clock64();
                    while (__hip_atomic_load(fp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < epoch) {
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
            }
            if (__syncthreads_or(gave_up)) return;   // the launch drains; agg_status reports the time-out
        }

        // ---- per-tile buffer descriptors and per-lane load offsets (bytes from the tile's A / B origin);
        // rows past the edge of the matrix fall outside the descriptor and load as zero
        const __amdgpu_buffer_rsrc_t a_rsrc =
            GROUPED ? make_rsrc(p.A, p.a_bytes)
                    : make_rsrc((from_local ? p.A_local + (long long)(m0 - p.local_lo) * p.lda : p.A + (long long)m0 * p.lda),
                                (unsigned)(min(BM, p.M - m0) * (int)p.lda * 2));
        const __amdgpu_buffer_rsrc_t b_rsrc =
            make_rsrc(p.B + (GROUPED ? (long long)expert * p.b_group_stride : 0ll) + (long long)n0 * p.ldb,
                      (unsigned)(min(BN, p.N - n0) * (int)p.ldb * 2));
        // unit i of this wave is unit u = wave + 4i of the stage: A units first, then B units
        unsigned ld_off[L];
#pragma unroll
        for (int i = 0; i < L; ++i) {
            const int u = wave + 4 * i;
            const int chunk = (u & 1) ? ld_chunk_odd : ld_chunk_even;
            if (4 * i < C_::A_UNITS) {
                if constexpr (GROUPED) {
                    // gathered row: the token of output row m0 + r; rows past the segment end get an offset outside
                    // the descriptor and load as zero
                    const int row = m0 + u * UNIT_ROWS + ld_row;
                    const int tok = row < m_lim ? (p.row_index ? p.row_index[row] : row) : -1;
                    ld_off[i] = tok >= 0 ? (unsigned)tok * (unsigned)(p.lda * 2) + (unsigned)(chunk * 16) : 0xFFFFFF00u;
                } else {
                    ld_off[i] = (unsigned)((u * UNIT_ROWS + ld_row) * (int)p.lda * 2 + chunk * 16);
                }
            } else
                ld_off[i] = (unsigned)(((u - C_::A_UNITS) * UNIT_ROWS + ld_row) * (int)p.ldb * 2 + chunk * 16);
        }

        // one global->LDS load: the i-th load of stage ks of this wave, into ring position pos (compile-time)
        // (the LDS address of this wave's quarter of ring position 0 is kept as a number the compiler cannot see
        // through: each load then takes one scalar add for its destination, instead of one live scalar register per
        // ring position)
        auto load_unit = [&](auto i_c, auto pos_c, int ks) {
            constexpr int i = decltype(i_c)::value, pos = decltype(pos_c)::value;
            constexpr bool is_a = 4 * i < C_::A_UNITS;      // the same for all four waves
            __builtin_amdgcn_raw_ptr_buffer_load_lds(is_a ? a_rsrc : b_rsrc, (lds_byte*)(unsigned long)(lds_wave + pos * 4096),
                                                     16, ld_off[i], ks * ROW_BYTES, 0, 0);
        };

        static_for<C_::ACC>([&](auto r) { acc_zero<decltype(r)::value>(); });

        if constexpr (MF == 16) {
            // ---- the 16x16x32 form.  Half-step h of a stage covers chunks 4h .. 4h+3 of the stage's rows (K = 32).  The A
            // fragments of the running half-step are fa[h], the next half-step's go into fa[1 - h] while it runs; the B
            // fragment of column block j lives in fb[j], which is free again after the MB16 MFMAs of group j and is
            // refilled at once with the next half-step's fragment j -- one set of B registers, not two.
            constexpr int MB16 = C_::MB16, NB16 = C_::NB16;
            constexpr int RW = C_::RW, PERIOD = C_::PERIOD;
            bf16x8 fa[2][MB16], fb[NB16];
            // A fragment i of this wave is 16-row block wave * MB16 + i of the tile's A rows; B fragment j is 16-row block
            // j of its B rows.  Two 16-row blocks share a ring position (the same load of all four waves = 32 rows).
            auto read_a = [&](auto i_c, auto base_c, auto h_c, int set) {
                constexpr int i = decltype(i_c)::value, base = decltype(base_c)::value, h = decltype(h_c)::value;
                const int rb = wave * MB16 + i;                  // wave-uniform
                int pos = base + (rb >> 1);
                if (pos >= RW) pos -= RW;
                fa[set][i] = *(lds_frag*)(unsigned long)(frb[h][0] + (unsigned)(pos * 4096 + (rb & 1) * 2048));
            };
            auto read_b = [&](auto j_c, auto base_c, auto h_c) {
                constexpr int j = decltype(j_c)::value, base = decltype(base_c)::value, h = decltype(h_c)::value;
                constexpr int pos = (base + C_::A_UNITS / 4 + j / 2) % RW;
                constexpr int off = pos * 4096 + (j & 1) * 2048;
                fb[j] = *(lds_frag*)(unsigned long)(frb[h][off >> 16] + (off & 0xFFFF));
            };

            // ---- prologue: the first P0 loads of the stream (stage 0, stage 1, the head of stage 2 ...); the main loop's
            // first groups continue the stream from there.  A stage past the end re-loads the last one: harmless, and
            // it keeps the count of outstanding loads the same on every path.
            static_for<C_::P0>([&](auto n_c) {
                constexpr int n = decltype(n_c)::value;
                load_unit(std::integral_constant<int, n % L>{}, std::integral_constant<int, n % RW>{}, min(n / L, KS - 1));
            });
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(C_::P0 - L));     // stage 0 has landed
            __builtin_amdgcn_s_barrier();
            static_for<MB16>([&](auto i_c) {
                read_a(i_c, std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, 0);
            });
            static_for<NB16>([&](auto j_c) {
                read_b(j_c, std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
            });

            // ---- main loop, PERIOD stages per pass so that ring positions are constants.  The MFMAs are volatile asm,
            // so memory operations keep their place between them: the order below is the schedule.  The B fragment
            // is the first MFMA operand, so accumulator block (i, j) holds the transposed 16x16 block.
            //
            // Stage ks: during half-step 0 every fragment of half-step 1 is read.  In half-step 1, after DLY groups (by
            // then the wave's last reads of stage ks are long back), the wave waits until its own loads of stage ks+1
            // have landed (RW - 2L younger ones may still be in flight) and meets the others at the barrier: all of
            // stage ks+1 is in LDS and nobody needs stage ks any more.  From there on the fragments of stage ks+1 are
            // read (those of the first DLY groups, held back until now, first), and the L ring positions of stage ks
            // are refilled: load n goes where load n - RW was; LH1 of them in the rest of this half-step, one per
            // group, the others in the first groups of the next stage.  They belong to stages ks+2 and later, so each
            // has about a stage of MFMA work to land.
            for (int ks0 = 0;; ks0 += PERIOD) {
                bool done = false;
                static_for<PERIOD>([&](auto ph_c) {
                    constexpr int ph = decltype(ph_c)::value;
                    if (done) return;
                    const int ks = ks0 + ph;
                    constexpr int base_cur = (ph * L) % RW;                              // ring base of stage ks
                    constexpr int base_next = ((ph + 1) * L) % RW;                       // of stage ks+1
                    constexpr int base_prev = (((ph + PERIOD - 1) % PERIOD) * L) % RW;   // of stage ks-1
                    asm volatile("" : "+s"(lds_wave), "+v"(frb[0][0]), "+v"(frb[0][1]), "+v"(frb[0][2]), "+v"(frb[1][0]),
                                 "+v"(frb[1][1]), "+v"(frb[1][2]));
                    static_for<2>([&](auto h_c) {
                        constexpr int h = decltype(h_c)::value;
                        // where the next half-step's fragments are
                        using next_base = std::integral_constant<int, h == 0 ? base_cur : base_next>;
                        using next_h = std::integral_constant<int, 1 - h>;
                        constexpr auto slots = C_::make_slots(h);
                        static_for<C_::NS>([&](auto s_c) {
                            constexpr int sl = decltype(s_c)::value;
                            constexpr int j = sl / MB16, i = sl % MB16;
                            mfma_acc16<i * NB16 + j>(fb[j], fa[h][i]);
                            if constexpr (h == 1 && sl == C_::SB) {
                                // stage ks+1 has landed for this wave (all but the RW - 2L youngest loads are back) and
                                // its own fragment reads of stage ks are back; after the barrier that holds for all waves
                                __builtin_amdgcn_s_waitcnt(vmcnt_imm(RW - 2 * L) & ~(0xF << 8));     // and lgkmcnt(0)
                                __builtin_amdgcn_s_barrier();
                            }
                            static_for<C_::PER_SLOT>([&](auto k_c) {
                                constexpr auto op = slots.op[sl][decltype(k_c)::value];
                                if constexpr (op.type == 1) {
                                    read_b(std::integral_constant<int, op.idx>{}, next_base{}, next_h{});
                                } else if constexpr (op.type == 2) {
                                    read_a(std::integral_constant<int, op.idx>{}, next_base{}, next_h{}, 1 - h);
                                } else if constexpr (op.type == 3) {
                                    // load op.idx of the batch released by this stage's barrier (h = 1) or by the
                                    // previous stage's (h = 0): stream index (stage * L) + RW + idx
                                    constexpr int jj = op.idx;
                                    if constexpr (h == 1)
                                        load_unit(std::integral_constant<int, (RW + jj) % L>{},
                                                  std::integral_constant<int, (base_cur + jj) % RW>{},
                                                  min(ks + (RW + jj) / L, KS - 1));
                                    else
                                        load_unit(std::integral_constant<int, (RW + jj) % L>{},
                                                  std::integral_constant<int, (base_prev + jj) % RW>{},
                                                  min(ks - 1 + (RW + jj) / L, KS - 1));
                                }
                            });
                        });
                    });
                    if (ks + 1 >= KS) done = true;
                });
                if (done) break;
            }
        } else {
            // two fragment sets, one per parity of the quarter-step.  Fragment f < MB is the A fragment of row
            // block f, fragment MB + j the B fragment of column block j.  The 32 rows of a fragment are the k-th
            // load of the stage (of all four waves), at ring position (base + k) mod RW, base = stage * L mod RW.
            bf16x8 fr[2][MB + NB];
            auto read_frag = [&](auto f_c, auto base_c, int h, int set) {
                constexpr int f = decltype(f_c)::value, base = decltype(base_c)::value;
                int pos;
                if constexpr (f < MB) {
                    pos = base + wave * MB + f;                  // wave-uniform
                    if (pos >= C_::RW) pos -= C_::RW;
                } else {
                    pos = (base + C_::A_UNITS / 4 + (f - MB)) % C_::RW;
                }
                fr[set][f] = *(const bf16x8*)(lds + pos * 4096 + fr_off[h]);
            };

            // ---- prologue: the first RW - L + LQ loads of the stream (stage 0, stage 1, the head of stage 2 ...);
            // the main loop's first quarter-steps continue the stream from there.  A stage past the end re-loads
            // the last one: harmless, and it keeps the count of outstanding loads the same on every path.
            constexpr int RW = C_::RW, PERIOD = C_::PERIOD, LQ = C_::LQ;
            static_for<RW - L + LQ>([&](auto n_c) {
                constexpr int n = decltype(n_c)::value;
                load_unit(std::integral_constant<int, n % L>{}, std::integral_constant<int, n % RW>{}, min(n / L, KS - 1));
            });
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(RW - 2 * L + LQ));     // stage 0 has landed
            __builtin_amdgcn_s_barrier();
            static_for<MB + NB>([&](auto f_c) { read_frag(f_c, std::integral_constant<int, 0>{}, 0, 0); });

            // ---- main loop, PERIOD stages per pass so that ring positions are constants.  The MFMAs are volatile
            // asm, so memory operations keep their place between them: the order below is the schedule.  Slot q of
            // a quarter-step works on column block q / MB, row block q % MB; the B fragment is the first MFMA
            // operand, so accumulator block (i, j) holds the transposed 32x32 block.
            //
            // Stage ks: quarter-steps 0..2 read ahead inside the stage; then every wave waits until its loads of
            // stage ks+1 have landed (RW - 2L younger ones may still be in flight) and meets the others at the
            // barrier -- all of stage ks+1 is in LDS and nobody needs stage ks any more; quarter-step 3 reads the
            // first fragments of stage ks+1.  Each barrier releases the L ring positions of stage ks: the next L
            // loads of the stream (load n goes where load n - RW was, and n - RW is a load of stage ks) are issued
            // LQ per quarter-step over the next three quarter-steps.  They belong to stages ks+2 and later, so each
            // has at least a whole stage of MFMA work to land.
            for (int ks0 = 0;; ks0 += PERIOD) {
                bool done = false;
                static_for<PERIOD>([&](auto ph_c) {
                    constexpr int ph = decltype(ph_c)::value;
                    if (done) return;
                    const int ks = ks0 + ph;
                    constexpr int base_cur = (ph * L) % RW;                          // ring base of stage ks
                    constexpr int base_next = ((ph + 1) * L) % RW;                   // of stage ks+1
                    constexpr int base_prev = (((ph + PERIOD - 1) % PERIOD) * L) % RW;   // of stage ks-1
                    static_for<QS>([&](auto h_c) {
                        constexpr int h = decltype(h_c)::value;
                        constexpr int set = h & 1;
                        static_for<C_::SLOTS>([&](auto q_c) {
                            constexpr int q = decltype(q_c)::value;
                            mfma_acc<(q % MB) * NB + q / MB>(fr[set][MB + q / MB], fr[set][q % MB]);
                            static_for<C_::QUOTA>([&](auto k_c) {
                                constexpr int o = q * C_::QUOTA + decltype(k_c)::value;
                                if constexpr (h == QS - 2) {
                                    // the quarter before the barrier issues no loads: its fragment reads go first, so
                                    // that they are back when the wave reaches the barrier
                                    if constexpr (o < C_::F)
                                        read_frag(std::integral_constant<int, o>{}, std::integral_constant<int, base_cur>{}, h + 1, 1 - set);
                                } else if constexpr (o < LQ) {
                                    // quarter 3 starts the batch released by this stage's barrier (j-th load of the
                                    // batch: stream index ks*L + RW + j); quarters 0 and 1 finish the batch released by
                                    // the previous stage's barrier
                                    if constexpr (h == QS - 1) {
                                        constexpr int j = o;
                                        if constexpr (j < L)
                                            load_unit(std::integral_constant<int, (RW + j) % L>{},
                                                           std::integral_constant<int, (base_cur + j) % RW>{},
                                                           min(ks + (RW + j) / L, KS - 1));
                                    } else {
                                        constexpr int j = (h + 1) * LQ + o;
                                        if constexpr (j < L)
                                            load_unit(std::integral_constant<int, (RW + j) % L>{},
                                                           std::integral_constant<int, (base_prev + j) % RW>{},
                                                           min(ks - 1 + (RW + j) / L, KS - 1));
                                    }
                                } else if constexpr (o - LQ < C_::F) {
                                    constexpr int f = o - LQ;
                                    if constexpr (h < QS - 1)
                                        read_frag(std::integral_constant<int, f>{}, std::integral_constant<int, base_cur>{}, h + 1, 1 - set);
                                    else
                                        read_frag(std::integral_constant<int, f>{}, std::integral_constant<int, base_next>{}, 0, 1 - set);
                                }
                            });
                        });
                        if constexpr (h == QS - 2) {
                            // stage ks+1 has landed for this wave (all but the RW - 2L youngest loads are back), its own
                            // fragment reads of this stage are back; after the barrier that holds for all waves
                            __builtin_amdgcn_s_waitcnt(vmcnt_imm(RW - 2 * L) & ~(0xF << 8));     // and lgkmcnt(0)
                            __builtin_amdgcn_s_barrier();
                        }
                    });
                    if (ks + 1 >= KS) done = true;
                });
                if (done) break;
            }
        }

        // ---- epilogue.  Accumulator block (i, j) is the transposed block: lane l holds output row
        // i*32 + l%32 and, in register v, column j*32 + 8*(v/4) + 4*(l/32) + v%4 -- four consecutive columns per
        // group of four registers.
        asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 7");     // the last MFMAs retire before the read-out
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));              // the last (redundant) loads have landed in LDS
        __syncthreads();                                       // and every wave is done with the ring
        {
            int lane_e = lane;
            asm volatile("" : "+v"(lane_e));     // keeps the address arithmetic below inside the tile loop
            const int row_w = m0 + wave * TM;    // first output row of this wave
            const int n_valid = min(BN, p.N - n0);      // columns of this tile inside the matrix
            // where a row of the output goes: C, or (GEMM-RS) the destination of its slice; nullptr = not stored
            auto row_ptr = [&](int row, int esz) -> char* {
                if (row < st_lo || row >= st_hi) return nullptr;
                if (!GROUPED && p.n_slices) {
                    const int w = row / p.slice_rows;
                    if (p.slice_dst[w])
                        return (char*)p.slice_dst[w] + ((long long)(row - w * p.slice_rows) * p.ldc_slice + n0) * esz;
                }
                return p.C ? (char*)p.C + ((long long)row * p.ldc + n0) * esz : nullptr;
            };
            auto epilogue = [&](auto tag) {
                using T = decltype(tag);                              // float or __bf16
                constexpr int esz = sizeof(T);
                typedef __attribute__((__vector_size__(4 * sizeof(T)))) T Tx4;
                typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;
                // whole 16-byte chunks of rows can be stored when the pointers allow it and the tile's valid width is
                // a whole number of chunks (always so for a full tile)
                const bool fast = p.c_vec_ok && (n_valid * esz) % 16 == 0;
                const int cpr_valid = n_valid * esz / 16;
                if constexpr (MF == 16 && esz == 4) {
                    if (fast) {
                        // fp32 output from 16x16 blocks: the four values a lane holds of a block are 16 consecutive
                        // bytes of an output row, and the four lanes that share a row cover 64 consecutive bytes --
                        // whole 64-byte sectors per store, so the values go from the registers straight to memory
                        // (neighbouring column blocks, stored back to back, complete the 128-byte lines in L2)
                        const int colq = 4 * (lane_e >> 4);
                        static_for<C_::MB16>([&](auto i_c) {
                            constexpr int i = decltype(i_c)::value;
                            char* dst = row_ptr(row_w + i * 16 + (lane_e & 15), esz);
                            if (dst) {
                                T* q = (T*)dst + colq;
                                static_for<C_::NB16>([&](auto j_c) {
                                    constexpr int j = decltype(j_c)::value;
                                    constexpr int r0 = (i * C_::NB16 + j) * 4;
                                    const float x0 = acc_read<r0>(), x1 = acc_read<r0 + 1>(), x2 = acc_read<r0 + 2>(),
                                                x3 = acc_read<r0 + 3>();
                                    if (n_valid == BN || colq + j * 16 < n_valid)
                                        __builtin_nontemporal_store(Tx4{(T)x0, (T)x1, (T)x2, (T)x3}, (Tx4*)(q + j * 16));
                                });
                            }
                        });
                        return;
                    }
                }
                if (fast) {
                    // stage 32 rows x BN columns per pass in this wave's own part of LDS, then move whole
                    // 16-byte chunks of rows to C: full cache lines per store instruction
                    constexpr int pitch = BN * esz + 16;
                    constexpr int cpr = BN * esz / 16;                // 16-byte chunks per row
                    constexpr int iters = (32 * cpr + 63) / 64;       // chunk c = lane + 64*it: row c / cpr, chunk c % cpr
                    unsigned char* stage = lds + wave * 32 * pitch;
                    unsigned char* wr = MF == 16 ? stage + (lane_e & 15) * pitch + 4 * (lane_e >> 4) * esz
                                                 : stage + (lane_e & 31) * pitch + 4 * (lane_e >> 5) * esz;
                    const int r_lane = lane_e / cpr, cc_lane = lane_e - r_lane * cpr;
                    static_for<MB>([&](auto i_c) {
                        constexpr int i = decltype(i_c)::value;
                        if constexpr (MF == 16) {
                            // 16x16 block (ib, j) of the pass: lane l holds row 16 ib + l%16, columns 16 j + 4 (l/16) + 0..3
                            static_for<2 * C_::NB16>([&](auto bj_c) {
                                constexpr int ib = decltype(bj_c)::value / C_::NB16, j = decltype(bj_c)::value % C_::NB16;
                                constexpr int r0 = ((2 * i + ib) * C_::NB16 + j) * 4;
                                const float x0 = acc_read<r0>(), x1 = acc_read<r0 + 1>(), x2 = acc_read<r0 + 2>(),
                                            x3 = acc_read<r0 + 3>();
                                *(Tx4*)(wr + ib * 16 * pitch + j * 16 * esz) = Tx4{(T)x0, (T)x1, (T)x2, (T)x3};
                            });
                        } else {
                            static_for<NB * 4>([&](auto jq_c) {
                                constexpr int j = decltype(jq_c)::value / 4, qd = decltype(jq_c)::value % 4;
                                constexpr int r0 = (i * NB + j) * 16 + qd * 4;
                                const float x0 = acc_read<r0>(), x1 = acc_read<r0 + 1>(), x2 = acc_read<r0 + 2>(),
                                            x3 = acc_read<r0 + 3>();
                                *(Tx4*)(wr + (j * 32 + qd * 8) * esz) = Tx4{(T)x0, (T)x1, (T)x2, (T)x3};
                            });
                        }
                        // the same wave wrote and reads: LDS keeps a wave's operations in order.  GRP chunks at a
                        // time: their LDS reads first (independent registers), then their stores.
                        const int row0 = row_w + i * 32;
                        // the 32 rows go to C, or (GEMM-RS) to the destination of their slice; a block that
                        // straddles a slice boundary takes the per-row route
                        const int rows_ok = min(32, st_hi - row0);
                        const int rows_lo = max(0, st_lo - row0);          // rows of the block before the first stored one
                        bool one_dst = true;          // all rows of the block have one destination matrix
                        char* base = p.C ? (char*)p.C + ((long long)row0 * p.ldc + n0) * esz : nullptr;
                        unsigned ld_bytes = (unsigned)(p.ldc * esz);
                        if (!GROUPED && p.n_slices && rows_ok > 0) {
                            const int w0 = row0 / p.slice_rows, w1 = (row0 + rows_ok - 1) / p.slice_rows;
                            one_dst = w0 == w1;
                            if (one_dst && p.slice_dst[w0]) {
                                base = (char*)p.slice_dst[w0] + ((long long)(row0 - w0 * p.slice_rows) * p.ldc_slice + n0) * esz;
                                ld_bytes = (unsigned)(p.ldc_slice * esz);
                            }
                        }
                        constexpr int GRP = 7;
                        int r = r_lane, cc = cc_lane;
                        if constexpr ((32 * cpr) % 64 == 0) {
                            // the common case -- all 32 rows inside the matrix (or segment) and bound for one
                            // destination -- has no per-lane conditions at all: every lane moves `iters` chunks
                            if (base && rows_ok >= 32 && rows_lo == 0 && n_valid == BN && one_dst) {
                                static_for<(iters + GRP - 1) / GRP>([&](auto g_c) {
                                    constexpr int it0 = decltype(g_c)::value * GRP;
                                    constexpr int n = (iters - it0 < GRP) ? iters - it0 : GRP;
                                    u32x4 val[n];
                                    unsigned off[n];
                                    static_for<n>([&](auto k_c) {
                                        constexpr int k = decltype(k_c)::value;
                                        off[k] = (unsigned)r * ld_bytes + (unsigned)cc * 16u;
                                        val[k] = *(const u32x4*)(stage + r * pitch + cc * 16);
                                        cc += 64 % cpr;
                                        r += 64 / cpr;
                                        const bool wrap = cc >= cpr;
                                        cc = wrap ? cc - cpr : cc;
                                        r = wrap ? r + 1 : r;
                                    });
                                    static_for<n>([&](auto k_c) {
                                        constexpr int k = decltype(k_c)::value;
                                        __builtin_nontemporal_store(val[k], (u32x4*)(base + off[k]));
                                    });
                                });
                                return;     // next row block
                            }
                        }
                        static_for<(iters + GRP - 1) / GRP>([&](auto g_c) {
                            constexpr int it0 = decltype(g_c)::value * GRP;
                            constexpr int n = (iters - it0 < GRP) ? iters - it0 : GRP;
                            u32x4 val[n];
                            int rs[n], ccs[n];
                            static_for<n>([&](auto k_c) {
                                constexpr int k = decltype(k_c)::value;
                                rs[k] = r;
                                ccs[k] = cc;
                                if (r < 32) val[k] = *(const u32x4*)(stage + r * pitch + cc * 16);
                                // next chunk of this lane: 64 chunks further on
                                cc += 64 % cpr;
                                r += 64 / cpr;
                                if (cc >= cpr) { cc -= cpr; r += 1; }
                            });
                            static_for<n>([&](auto k_c) {
                                constexpr int k = decltype(k_c)::value;
                                if (one_dst) {
                                    if (base && rs[k] < rows_ok && rs[k] >= rows_lo && ccs[k] < cpr_valid) {
                                        // C is not read again by this kernel: streaming stores keep it from
                                        // displacing the A and B lines that are
                                        __builtin_nontemporal_store(val[k], (u32x4*)(base + (unsigned)rs[k] * ld_bytes + (unsigned)ccs[k] * 16u));
                                    }
                                } else {
                                    char* dst = (rs[k] < 32 && ccs[k] < cpr_valid) ? row_ptr(row0 + rs[k], esz) : nullptr;
                                    if (dst) *(u32x4*)(dst + ccs[k] * 16) = val[k];
                                }
                            });
                        });
                    });
                } else {
                    // edge tiles and unaligned outputs: one element at a time, constant offsets from one row pointer
                    if constexpr (MF == 16) {
                        static_for<C_::MB16>([&](auto i_c) {
                            constexpr int i = decltype(i_c)::value;
                            char* dst = row_ptr(row_w + i * 16 + (lane_e & 15), esz);
                            const int col0 = n0 + 4 * (lane_e >> 4);
                            T* q = (T*)dst + 4 * (lane_e >> 4);
                            static_for<C_::NB16 * 4>([&](auto jv_c) {
                                constexpr int j = decltype(jv_c)::value / 4, v = decltype(jv_c)::value % 4;
                                constexpr int off = j * 16 + v;
                                const float x = acc_read<(i * C_::NB16 + j) * 4 + v>();
                                if (dst && col0 + off < p.N) q[off] = (T)x;
                            });
                        });
                    } else {
                    static_for<MB>([&](auto i_c) {
                        constexpr int i = decltype(i_c)::value;
                        char* dst = row_ptr(row_w + i * 32 + (lane_e & 31), esz);
                        const int col0 = n0 + 4 * (lane_e >> 5);
                        T* q = (T*)dst + 4 * (lane_e >> 5);
                        static_for<NB * 16>([&](auto jv_c) {
                            constexpr int j = decltype(jv_c)::value / 16, v = decltype(jv_c)::value % 16;
                            constexpr int off = j * 32 + 8 * (v >> 2) + (v & 3);
                            const float x = acc_read<(i * NB + j) * 16 + v>();
                            if (dst && col0 + off < p.N) q[off] = (T)x;
                        });
                    });
                    }
                }
            };
            if (p.c_is_f32) epilogue(float{}); else epilogue(__bf16{});
        }

        // GEMM-RS: count this tile for every chunk of every slice it touches; the last tile of a chunk raises the
        // chunk's signal (the notify of Algorithm 3: those rows are complete where their reducer will read them)
        if (!GROUPED && p.n_slices && p.slice_ctr) {
            const int w_lo = m0 / p.slice_rows, w_hi = (min(m0 + BM, p.M) - 1) / p.slice_rows;
            bool any = false;
            for (int w = w_lo; w <= w_hi; ++w) any = any || p.slice_flag[w] != nullptr;
            if (any) {
                __builtin_amdgcn_s_waitcnt(0);   // this wave's stores of the tile have reached L2 ...
                __syncthreads();                 // ... and so have every other wave's, before thread 0 publishes them
                if (tid == 0) {
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
                    const int m_end = min(m0 + BM, p.M);
                    for (int w = w_lo; w <= w_hi; ++w) {
                        if (!p.slice_flag[w]) continue;
                        const int s0 = w * p.slice_rows;                       // first row of slice w
                        const int c_lo = (max(m0, s0) - s0) / p.chunk_rows;
                        const int c_hi = (min(m_end, s0 + p.slice_rows) - 1 - s0) / p.chunk_rows;
                        for (int c = c_lo; c <= c_hi; ++c) {
                            // tiles that touch these rows: their m-tiles times all n-tiles
                            const int r0 = s0 + c * p.chunk_rows;
                            const int mt_lo = r0 / BM, mt_hi = (r0 + p.chunk_rows - 1) / BM;
                            const int target = (mt_hi - mt_lo + 1) * p.tiles_n;
                            int* ctr = p.slice_ctr + w * p.slice_chunks + c;
                            const int prev = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
                            if (prev == target - 1) {
                                __hip_atomic_store(ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                                __hip_atomic_store(p.slice_flag[w] + c * kSignalStride, epoch, __ATOMIC_RELEASE,
                                                   __HIP_MEMORY_SCOPE_AGENT);
                            }
                        }
                    }
                }
            }
        }

        // the stage buffers are reused by the next tile: every wave must be done with its staging reads first.
        // The C stores need not be waited for: the next tile's waits count them as well, which only makes
        // those waits stricter.
        __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0) only (vmcnt and expcnt fields at their no-wait maximum)
        __builtin_amdgcn_s_barrier();
    }
#else
    (void)p;
#endif
}

template <int BM, int BN, bool GROUPED, int MF>
static hipError_t launch_cfg(const GemmParams& p, int grid, hipStream_t stream)
{
    using C_ = Cfg<BM, BN>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)gemm_kernel<BM, BN, GROUPED, MF>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C_::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((gemm_kernel<BM, BN, GROUPED, MF>), dim3(grid), dim3(256), C_::LDS_BYTES, stream, p);
    return hipGetLastError();
}

}  // namespace agg

// One translation unit per tile configuration instantiates the plain and the grouped kernel of that configuration
// (gemm_inst_*.hip), so that they compile side by side.
#define AGG_GEMM_INSTANCE(BM, BN, MF)                                                                        \
    namespace agg {                                                                                          \
    hipError_t launch_gemm_##BM##x##BN##_mf##MF(const GemmParams& p, bool grouped, int grid, hipStream_t s)  \
    {                                                                                                        \
        return grouped ? launch_cfg<BM, BN, true, MF>(p, grid, s) : launch_cfg<BM, BN, false, MF>(p, grid, s); \
    }                                                                                                        \
    }

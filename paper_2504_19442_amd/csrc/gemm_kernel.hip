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
// (buffer_load_dwordx4 ... lds, 16 bytes per lane) through a ring of NS stages, so NS-1 steps of loads are
// in flight while one is computed.  Rows are 64 bytes in LDS; the 16-byte chunk c of row r sits in slot
// c ^ ((r >> 2) & 3), which makes the ds_read_b128 operand fetches bank-conflict free.  Each wave owns
// BM/4 rows and all BN columns of the tile and feeds v_mfma_f32_32x32x16_bf16 from register sets of
// fragments that are refilled one half-step ahead of their use.  One workgroup barrier per step.  The
// fragment reads and global->LDS loads of a step are dealt out one per MFMA (a wave issues in order and a
// memory instruction is slow to issue, so bunches of them between two MFMAs starve the matrix pipe).
// The MFMA computes the transposed block (B fragment as first operand), so that a lane ends up holding
// four consecutive columns of one output row; the epilogue stages each wave's rows through LDS and
// stores them to C as whole 16-byte row chunks.
//
// Registers: the fp32 accumulators live in accumulator registers a0..a(MB*NB*16-1) that only the inline
// asm of this file touches (MFMA, zeroing, read-out); the compiler allocates the ordinary registers and is
// capped so that the kernel takes 448 of the 512 registers of a SIMD.  The 64 left over are what lets one
// wave of a small kernel (the producer's copy waves, the reducer) run beside a consumer wave on every
// SIMD: communication and computation share all CUs instead of splitting them (Section 3.8).
#include "agg_internal.h"

#include <type_traits>
#include <utility>

namespace agg {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;

#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

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
#ifdef AGG_EXP_NO_MFMA
    asm volatile("; no mfma %2 %3" ::"v"(a), "v"(b), "n"(BLK * 16), "n"(BLK * 16 + 15));
#else
    asm volatile("v_mfma_f32_32x32x16_bf16 a[%2:%3], %0, %1, a[%2:%3]" ::"v"(a), "v"(b), "n"(BLK * 16), "n"(BLK * 16 + 15));
#endif
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

constexpr int BK = 32;                 // bf16 per K-step
constexpr int ROW_BYTES = BK * 2;      // 64-byte rows in LDS
constexpr int UNIT_ROWS = 16;          // one wave-wide 16-byte-per-lane load covers 16 rows

template <int BM, int BN, int NS>
struct Cfg {
    static constexpr int TM = BM / 4;            // rows per wave
    static constexpr int MB = TM / 32;           // 32x32 blocks per wave, M direction
    static constexpr int NB = BN / 32;           // and N direction
    static constexpr int ACC = MB * NB * 16;     // accumulator registers per lane
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
    static_assert(ACC == 64 || ACC == 128 || ACC == 224 || ACC == 256, "add a reservation line for this accumulator count");
    // MFMA slots of one K-step: [0, SLOTS_A) before the barrier, then the rest of half-step 0, then half-step 1
    // (slots [SLOTS/2, SLOTS)).  A wave issues in order, and a memory instruction takes long enough to issue
    // that more than one or two of them between two MFMAs leaves the matrix pipe idle; so every slot gets at
    // most QUOTA memory instructions.  First half of the step: the F = MB+NB fragment reads of half-step 1,
    // then L1 of the step's global->LDS loads; second half: the F fragment reads of the next step's
    // half-step 0, then the remaining loads.
    static constexpr int H = NB / 2;
    static constexpr int SLOTS = 2 * MB * NB;
    static constexpr int SLOTS_A = MB * H;
    static constexpr int F = MB + NB;
    static constexpr int QUOTA = (2 * F + L + SLOTS - 1) / SLOTS;
    static constexpr int CAP = (SLOTS / 2) * QUOTA;              // memory instructions per half
    static constexpr int L1 = (L < CAP - F) ? L : CAP - F;       // loads issued in the first half
    static_assert(CAP >= F && F + (L - L1) <= CAP, "memory instructions do not fit the slots");
    static_assert(F / QUOTA >= SLOTS_A, "the first load of a step must come after the barrier");
    // epilogue staging: each wave stages 32 rows x BN columns at a time
    static constexpr int PITCH_BF16 = BN * 2 + 16;
    static constexpr int PITCH_F32 = BN * 4 + 16;
    static_assert(4 * 32 * PITCH_F32 <= LDS_BYTES, "epilogue staging does not fit in the ring");
};

template <int BM, int BN, int NS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_num_vgpr(224))) void gemm_kernel(const GemmParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)    // the body names gfx950 registers; the host pass only needs the launch stub
    using C_ = Cfg<BM, BN, NS>;
    constexpr int MB = C_::MB, NB = C_::NB, L = C_::L, FULL = C_::FULL, TM = C_::TM;
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
#ifndef AGG_EXP_NO_ACQ
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
#endif
            if (__syncthreads_or(gave_up)) return;   // the launch drains; agg_status reports the time-out
        }

        // ---- per-tile buffer descriptors and per-lane load offsets (bytes from the tile's A / B origin);
        // rows past the edge of the matrix fall outside the descriptor and load as zero
        const __amdgpu_buffer_rsrc_t a_rsrc =
            make_rsrc(p.A + (long long)m0 * p.lda, (unsigned)(min(BM, p.M - m0) * (int)p.lda * 2));
        const __amdgpu_buffer_rsrc_t b_rsrc =
            make_rsrc(p.B + (long long)n0 * p.ldb, (unsigned)(min(BN, p.N - n0) * (int)p.ldb * 2));
        unsigned ld_off[L];
#pragma unroll
        for (int i = 0; i < L; ++i) {
            const int u = (i < FULL) ? wave + 4 * i : 4 * FULL + (wave >> 1);
            if (u < C_::A_UNITS)
                ld_off[i] = (unsigned)((u * UNIT_ROWS + ld_row) * (int)p.lda * 2 + ld_chunk * 16);
            else
                ld_off[i] = (unsigned)(((u - C_::A_UNITS) * UNIT_ROWS + ld_row) * (int)p.ldb * 2 + ld_chunk * 16);
        }

        // one global->LDS load (unit i of this wave) of K-step kt into stage st
        auto load_unit = [&](int i, int st, int kt) {
            const int u = (i < FULL) ? wave + 4 * i : 4 * FULL + (wave >> 1);
            // whether unit i of this wave is an A or a B unit is the same for all four waves
            const bool is_a = ((i < FULL) ? 4 * i : 4 * FULL) < C_::A_UNITS;
#ifdef AGG_EXP_SAME_M0
            unsigned char* dst = lds + st * C_::STAGE_BYTES + (u & 3) * 1024;
#else
            unsigned char* dst = lds + st * C_::STAGE_BYTES + u * 1024;
#endif
#if defined(AGG_EXP_MB1)
            // microbenchmark-like addressing, step 1: one descriptor, private rows per wave, 2 KiB window
            __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, LDS_PTR(dst), 16,
                                                     (unsigned)((wave * 64 + i * 16 + ld_row) * 16384 + ld_chunk * 16) % (3u << 20),
                                                     (kt & 31) * ROW_BYTES, 0, 0);
#elif defined(AGG_EXP_MB2)
            // step 2: real descriptors and offsets, but the K offset cycles inside a 2 KiB window
            __builtin_amdgcn_raw_ptr_buffer_load_lds(is_a ? a_rsrc : b_rsrc, LDS_PTR(dst), 16, ld_off[i],
                                                     (kt & 31) * ROW_BYTES, 0, 0);
#elif defined(AGG_EXP_MB3)
            // step 3: real K offsets, one descriptor
            __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, LDS_PTR(dst), 16,
                                                     (unsigned)((wave * 64 + i * 16 + ld_row) * 16384 + ld_chunk * 16) % (3u << 20),
                                                     kt * ROW_BYTES, 0, 0);
#elif defined(AGG_EXP_MB4)
            // real offsets, one descriptor
            __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, LDS_PTR(dst), 16, ld_off[i], kt * ROW_BYTES, 0, 0);
#elif defined(AGG_EXP_MB5)
            // two descriptors, wave-private rows
            __builtin_amdgcn_raw_ptr_buffer_load_lds(is_a ? a_rsrc : b_rsrc, LDS_PTR(dst), 16,
                                                     (unsigned)((wave * 64 + i * 16 + ld_row) * 16384 + ld_chunk * 16) % (3u << 20),
                                                     kt * ROW_BYTES, 0, 0);
#elif defined(AGG_EXP_MB6)
            // two descriptors, real row ranges, rows contiguous per wave
            {
                const int unit = is_a ? wave * 4 + i : min(wave * 4 + (i - 4), C_::B_UNITS - 1);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(is_a ? a_rsrc : b_rsrc, LDS_PTR(dst), 16,
                                                         (unsigned)((unit * 16 + ld_row) * 16384 + ld_chunk * 16),
                                                         kt * ROW_BYTES, 0, 0);
            }
#elif defined(AGG_EXP_MB7)
            // real pattern but B rows taken from the A tile region +256 rows (distinct lines, A descriptor)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, LDS_PTR(dst), 16, ld_off[i] + (is_a ? 0u : 0u),
                                                     kt * ROW_BYTES + (is_a ? 0 : 8192 * 2 * 0), 0, 0);
#elif defined(AGG_EXP_SAME_K)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(is_a ? a_rsrc : b_rsrc, LDS_PTR(dst), 16, ld_off[i],
                                                     (kt & 1) * ROW_BYTES, 0, 0);
#elif defined(AGG_EXP_LOAD_VGPR)
            typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4_;
            u32x4_ v_ = __builtin_amdgcn_raw_buffer_load_b128(is_a ? a_rsrc : b_rsrc, ld_off[i], kt * ROW_BYTES, 0);
            asm volatile("" ::"v"(v_));
            (void)dst;
#else
            __builtin_amdgcn_raw_ptr_buffer_load_lds(is_a ? a_rsrc : b_rsrc, LDS_PTR(dst), 16, ld_off[i],
                                                     kt * ROW_BYTES, 0, 0);
#endif
        };

        // three fragment sets: sets 0 and 1 alternate for half-step 0 (the next step's is fetched while the
        // current one is still being used), set 2 serves half-step 1.  Fragment f < MB is the A fragment of
        // row block f, fragment MB + j the B fragment of column block j.
        bf16x8 fr[3][MB + NB];
        auto read_frag = [&](int f, int st, int s, int set) {
            const unsigned char* src = lds + st * C_::STAGE_BYTES + fr_off[s] +
                                       (f < MB ? (wave * TM + f * 32) * ROW_BYTES : (BM + (f - MB) * 32) * ROW_BYTES);
            fr[set][f] = *(const bf16x8*)src;
        };

#ifdef AGG_EXP_TIMING
        const long long tt0 = __builtin_readcyclecounter();
#endif
        static_for<C_::ACC>([&](auto r) { acc_zero<decltype(r)::value>(); });

        // ---- prologue: NS-1 stages in flight (steps past the end re-load the last step: harmless, and it
        // keeps the number of outstanding loads per wave the same on every path)
#pragma unroll
        for (int st = 0; st < NS - 1; ++st)
#pragma unroll
            for (int i = 0; i < L; ++i) load_unit(i, st, min(st, KT - 1));
        __builtin_amdgcn_s_waitcnt(vmcnt_imm((NS - 2) * L));
        __builtin_amdgcn_s_barrier();
#pragma unroll
        for (int f = 0; f < MB + NB; ++f) read_frag(f, 0, 0, 0);

        // experiment switches (never defined in the product build): drop work from the main loop to see what it costs
#ifdef AGG_EXP_NO_LDSREAD
#define LOOP_READ_FRAG(...) ((void)0)
#else
#define LOOP_READ_FRAG(...) read_frag(__VA_ARGS__)
#endif
#ifdef AGG_EXP_NO_GLOAD
#define LOOP_LOAD_UNIT(...) ((void)0)
#else
#define LOOP_LOAD_UNIT(...) load_unit(__VA_ARGS__)
#endif
        // ---- main loop, unrolled over the ring so that stage and set indices are constants.  The MFMAs are
        // volatile asm, so memory operations keep their place between them: the interleaving below is the
        // schedule.  Slot q of a half-step works on column block q / MB, row block q % MB; the B fragment is
        // the first MFMA operand, so accumulator block (i, j) holds the transposed 32x32 block.
#ifdef AGG_EXP_TIMING
        const long long tt1 = __builtin_readcyclecounter();
#endif
        for (int kt0 = 0;; kt0 += NS) {
            bool done = false;
            static_for<NS>([&](auto st_c) {
                constexpr int st = decltype(st_c)::value;
                constexpr int cur = st & 1, nxt = (st + 1) & 1;
                if (done) return;
                const int kt = kt0 + st;
                const int kt_load = min(kt + NS - 1, KT - 1);
                // the memory instructions that follow the MFMA of slot `slot`
                auto mem_after = [&](auto slot_c) {
                    constexpr int slot = decltype(slot_c)::value;
                    constexpr bool second = slot >= C_::SLOTS / 2;
                    static_for<C_::QUOTA>([&](auto k_c) {
                        constexpr int o = (slot % (C_::SLOTS / 2)) * C_::QUOTA + decltype(k_c)::value;
                        if constexpr (o < C_::F) {
                            // fragment reads: half-step 1 of this step, or half-step 0 of the next step
                            if constexpr (!second) LOOP_READ_FRAG(o, st, 1, 2);
                            else LOOP_READ_FRAG(o, (st + 1) % NS, 0, nxt);
                        } else {
                            // global->LDS loads of step kt+NS-1 into the stage every wave finished reading
                            // before the barrier of this step
                            constexpr int i = (second ? C_::L1 : 0) + o - C_::F;
                            if constexpr (i < (second ? L : C_::L1)) LOOP_LOAD_UNIT(i, (st + NS - 1) % NS, kt_load);
                        }
                    });
                };
                static_for<C_::SLOTS>([&](auto q_c) {
                    constexpr int slot = decltype(q_c)::value;
                    constexpr int set = slot < C_::SLOTS / 2 ? cur : 2;
                    constexpr int q = slot % (C_::SLOTS / 2);       // column block q / MB, row block q % MB
                    mfma_acc<(q % MB) * NB + q / MB>(fr[set][MB + q / MB], fr[set][q % MB]);
                    mem_after(q_c);
                    if constexpr (slot == C_::SLOTS_A - 1) {
#ifndef AGG_EXP_NO_BARRIER
                        // stage kt+1 has landed for this wave once at most the younger stages are outstanding;
                        // after the barrier it has landed for all waves, and all waves are done with stage kt-1
                        __builtin_amdgcn_s_waitcnt(vmcnt_imm((NS - 3) * L));
                        __builtin_amdgcn_s_barrier();
#endif
                    }
                });
                if (kt + 1 >= KT) done = true;
            });
            if (done) break;
        }

        // ---- epilogue.  Accumulator block (i, j) is the transposed block: lane l holds output row
        // i*32 + l%32 and, in register v, column j*32 + 8*(v/4) + 4*(l/32) + v%4 -- four consecutive columns per
        // group of four registers.
#ifdef AGG_EXP_TIMING
        const long long tt2 = __builtin_readcyclecounter();
#endif
        asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 7");     // the last MFMAs retire before the read-out
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));              // the last (redundant) loads have landed in LDS
        __syncthreads();                                       // and every wave is done with the ring
        {
            int lane_e = lane;
            asm volatile("" : "+v"(lane_e));     // keeps the address arithmetic below inside the tile loop
            const int row_w = m0 + wave * TM;    // first output row of this wave
            const bool fast = p.c_vec_ok && n0 + BN <= p.N;
            // where a row of the output goes: C, or (GEMM-RS) this rank's own slot; nullptr = not stored
            auto row_ptr = [&](int row, int esz) -> char* {
                if (row >= p.M) return nullptr;
                if (p.C_own && row >= p.own_lo && row < p.own_hi)
                    return (char*)p.C_own + ((long long)(row - p.own_lo) * p.ldc_own + n0) * esz;
                return p.C ? (char*)p.C + ((long long)row * p.ldc + n0) * esz : nullptr;
            };
            auto epilogue = [&](auto tag) {
                using T = decltype(tag);                              // float or __bf16
                constexpr int esz = sizeof(T);
                typedef __attribute__((__vector_size__(4 * sizeof(T)))) T Tx4;
                typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;
                if (fast) {
                    // stage 32 rows x BN columns per pass in this wave's own part of LDS, then move whole
                    // 16-byte chunks of rows to C: full cache lines per store instruction
                    constexpr int pitch = BN * esz + 16;
                    constexpr int cpr = BN * esz / 16;                // 16-byte chunks per row
                    unsigned char* stage = lds + wave * 32 * pitch;
                    unsigned char* wr = stage + (lane_e & 31) * pitch + 4 * (lane_e >> 5) * esz;
                    static_for<MB>([&](auto i_c) {
                        constexpr int i = decltype(i_c)::value;
                        static_for<NB * 4>([&](auto jq_c) {
                            constexpr int j = decltype(jq_c)::value / 4, qd = decltype(jq_c)::value % 4;
                            constexpr int r0 = (i * NB + j) * 16 + qd * 4;
                            const float x0 = acc_read<r0>(), x1 = acc_read<r0 + 1>(), x2 = acc_read<r0 + 2>(),
                                        x3 = acc_read<r0 + 3>();
                            *(Tx4*)(wr + (j * 32 + qd * 8) * esz) = Tx4{(T)x0, (T)x1, (T)x2, (T)x3};
                        });
                        // the same wave wrote and reads: LDS keeps a wave's operations in order
                        for (int c = lane_e; c < 32 * cpr; c += 64) {
                            const int r = c / cpr, cc = c - r * cpr;
                            const u32x4 val = *(const u32x4*)(stage + r * pitch + cc * 16);
                            char* dst = row_ptr(row_w + i * 32 + r, esz);
                            if (dst) *(u32x4*)(dst + cc * 16) = val;
                        }
                    });
                } else {
                    // edge tiles and unaligned outputs: one element at a time, constant offsets from one row pointer
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
            };
            if (p.c_is_f32) epilogue(float{}); else epilogue(__bf16{});
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
#ifdef AGG_EXP_TIMING
        if (tid == 0 && (g == 0 || g == 100)) {
            const long long tt3 = __builtin_readcyclecounter();
            long long* dbg = (long long*)(p.err + 8) + (g ? 4 : 0);
            dbg[0] = tt1 - tt0; dbg[1] = tt2 - tt1; dbg[2] = tt3 - tt2; dbg[3] = KT;
        }
#endif
    }
#else
    (void)p;
#endif
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
        default: return launch_cfg<128, 128, 6>(p, grid, stream);
    }
}

}  // namespace agg

// C ABI of libagg.so: argument checks, context bookkeeping and launches.  No arithmetic of the
// method happens on the host; every step runs in the HIP kernels of this library.
#include "agg_internal.h"

#include <algorithm>
#include <vector>

#include <new>

using namespace agg;

namespace {

inline int hip_fail(hipError_t e)
{
    if (e == hipSuccess) return AGG_OK;
    (void)hipGetLastError();
    return e == hipErrorOutOfMemory ? AGG_ERR_NOMEM : AGG_ERR_HIP;
}

#define HIP_TRY(x)                         \
    do {                                   \
        int rc_ = hip_fail((x));           \
        if (rc_ != AGG_OK) return rc_;     \
    } while (0)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline long long wait_ticks(const agg_ctx* c)
{
    return (long long)((double)c->wall_khz * (double)c->wait_limit_us / 1000.0);
}

// Pick the tile shape with the smallest estimated time: waves of tiles over the CUs times the cost of a
// tile (its area over a rough efficiency of the shape).
int choose_tile(const agg_ctx* c, int M, int N)
{
    if (c->tile_config >= 0) return c->tile_config;
    // measured rates per flop relative to the large shapes (70B shape, GEMM alone): 128x256 0.86, 128x128 0.78
    const int cand[4] = {TILE_256x224, TILE_256x256, TILE_128x256, TILE_128x128};
    const double eff[4] = {1.0, 1.0, 0.86, 0.75};
    int best = cand[0];
    double best_cost = 1e300;
    for (int i = 0; i < 4; ++i) {
        const TileShape t = tile_shape(cand[i]);
        const long long tiles = (long long)((M + t.bm - 1) / t.bm) * ((N + t.bn - 1) / t.bn);
        const long long waves = (tiles + c->num_cus - 1) / c->num_cus;
        const double cost = (double)waves * t.bm * t.bn / eff[i];
        if (cost < best_cost) {
            best_cost = cost;
            best = cand[i];
        }
    }
    // the 16x16x32 form of the main loop: the same work at a lower power per flop, so the chip holds a higher clock
    // (measured 5 to 8 % faster on every shape); the 32x32x16 form stays selectable (configurations 0 to 3)
    return best | TILE_K32;
}

// Fill the schedule fields: panels of `rows_per_shard` rows starting at the panel of `first_row`.
void fill_schedule(GemmParams& p, int cfg, int rows_per_shard, int first_row)
{
    const TileShape t = tile_shape(cfg);
    p.tiles_m = (p.M + t.bm - 1) / t.bm;
    p.tiles_n = (p.N + t.bn - 1) / t.bn;
    int pm = rows_per_shard / t.bm;
    if (pm < 1) pm = 1;
    if (pm > 32) pm = 32;
    p.panel_m = pm;
    p.group_n = 32 / pm > 0 ? 32 / pm : 1;
    p.m_tile_start = p.tiles_m > 0 ? (first_row / t.bm) % p.tiles_m : 0;
}

int check_gemm_operands(int M, int N, int K, const void* B, int ldb, int b_layout, const void* C, int ldc, int c_dtype)
{
    if (M < 0 || N < 0 || K < 0) return AGG_ERR_INVALID_ARG;
    if (c_dtype != AGG_BF16 && c_dtype != AGG_F32) return AGG_ERR_INVALID_ARG;
    if (b_layout != AGG_B_NK && b_layout != AGG_B_KN) return AGG_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return AGG_OK;
    if (!B || !C) return AGG_ERR_INVALID_ARG;
    if (K == 0 || K % 64 != 0 || K > (1 << 21)) return AGG_ERR_UNSUPPORTED_SHAPE;
    if (ldb < (b_layout == AGG_B_NK ? K : N) || ldc < N) return AGG_ERR_INVALID_ARG;
    if (b_layout == AGG_B_NK && (ldb % 8 != 0 || !aligned16(B))) return AGG_ERR_MISALIGNED;
    if (b_layout == AGG_B_KN && reinterpret_cast<uintptr_t>(B) % 2 != 0) return AGG_ERR_MISALIGNED;
    if (reinterpret_cast<uintptr_t>(C) % (c_dtype == AGG_F32 ? 4 : 2) != 0) return AGG_ERR_MISALIGNED;
    return AGG_OK;
}

// The GEMM kernel reads B as [N][K].  A B given as [K][N] is transposed first, on the GEMM's stream, into a buffer
// of the context that agg_reserve_b_kn has sized beforehand: the call itself allocates nothing.  Callers whose
// weights do not change should store them as [N][K] and save the pass (2 x N x K x 2 bytes of traffic per call).
int resolve_b(agg_ctx* c, const void* B, int ldb, int b_layout, int N, int K, hipStream_t stream, const uint16_t** B_nk,
              long long* ld_nk)
{
    if (b_layout == AGG_B_NK) {
        *B_nk = (const uint16_t*)B;
        *ld_nk = ldb;
        return AGG_OK;
    }
    if (c->b_nk_elems < (size_t)N * K) return AGG_ERR_NOT_RESERVED;
    // the buffer is one per context: a call on another stream than the last one that used it first waits (on the
    // device) for that one's GEMM, so that two such calls can never read each other's transposed B
    if (c->b_nk_in_use && stream != c->b_nk_stream) HIP_TRY(hipStreamWaitEvent(stream, c->b_nk_free, 0));
    HIP_TRY(launch_transpose_kn((const uint16_t*)B, ldb, K, N, c->b_nk, stream));
    *B_nk = c->b_nk;
    *ld_nk = K;
    return AGG_OK;
}

// After the launch of a GEMM that reads the context's transposed copy of B: mark where the buffer becomes free again.
int b_kn_launched(agg_ctx* c, int b_layout, hipStream_t stream)
{
    if (b_layout != AGG_B_KN) return AGG_OK;
    HIP_TRY(hipEventRecord(c->b_nk_free, stream));
    c->b_nk_stream = stream;
    c->b_nk_in_use = 1;
    return AGG_OK;
}

// ---- device memory that no call allocates: a fixed array in the library's image, one copy per GPU, used by
// ag_moe_gemm_static for the MoE routing's control block and the grouped GEMM's tile table.  Host code never uses the array's name as an
// address: the device address is looked up once per context (symm_alloc, with the context's device current).
constexpr size_t kStaticTabOffset = kMoeCtrlBytes;         // the routing's control block first, the table after it
constexpr size_t kStaticTabEntries = 32760;
constexpr size_t kStaticScratchBytes = kStaticTabOffset + kStaticTabEntries * sizeof(MoeTile);   // 1088 KiB
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Upper bound of the grouped GEMM's tile table over all tile configurations: sum over experts of
// ceil(rows / bm) <= P / bm + E, times the n-tiles, for the smallest tile (128 x 128).
long long moe_table_bound(long long P, int E, int N) { return (P / 128 + E) * ((N + 127) / 128); }

// The producer stream must run side by side with the consumer stream: streams that the runtime has put on one
// hardware queue run their kernels one after the other.  Which queue a new stream gets cannot be asked for, so it
// is tried out: a one-thread kernel on the consumer stream waits (for at most 0.5 ms) for a word that a one-thread
// kernel on the candidate stream sets.  The first candidate whose kernel gets through while the other still waits
// is kept.  If none of eight does, the last one is kept: the library then still works when the producer is launched
// first, as the interface asks of callers with streams of their own.
int pick_concurrent_stream(agg_ctx* c)
{
    constexpr int kTries = 8;
    hipStream_t cand[kTries] = {nullptr};
    int* word = c->err + 32;              // two words of the context's bookkeeping block
    int rc = AGG_OK, chosen = -1, made = 0;
    for (int i = 0; i < kTries && chosen < 0; ++i) {
        if ((rc = hip_fail(hipStreamCreateWithFlags(&cand[i], hipStreamNonBlocking))) != AGG_OK) break;
        made = i + 1;
        if ((rc = hip_fail(hipMemset(word, 0, 2 * sizeof(int)))) != AGG_OK) break;
        if ((rc = hip_fail(hipDeviceSynchronize())) != AGG_OK) break;
        if ((rc = hip_fail(launch_signal_probe(word, 1, c->wall_khz / 2, word + 1, c->consumer_stream))) != AGG_OK) break;
        if ((rc = hip_fail(launch_signal_set(word, 1, nullptr, cand[i]))) != AGG_OK) break;
        if ((rc = hip_fail(hipDeviceSynchronize())) != AGG_OK) break;
        int seen = 0;
        if ((rc = hip_fail(hipMemcpy(&seen, word + 1, sizeof seen, hipMemcpyDeviceToHost))) != AGG_OK) break;
        if (seen == 1) chosen = i;
    }
    if (rc == AGG_OK && chosen < 0) chosen = made - 1;
    for (int i = 0; i < made; ++i)
        if (i != chosen || rc != AGG_OK) (void)hipStreamDestroy(cand[i]);
    if (rc != AGG_OK) return rc;
    c->producer_stream = cand[chosen];
    (void)hipMemset(word, 0, 2 * sizeof(int));
    return AGG_OK;
}

}  // namespace

extern "C" {

int symm_alloc(agg_ctx** out, int world_size, int rank, size_t shard_bytes, int n_signals)
{
    if (!out || world_size < 1 || world_size > kMaxWorld || rank < 0 || rank >= world_size) return AGG_ERR_INVALID_ARG;
    if (n_signals < world_size || n_signals % world_size != 0 || n_signals > (1 << 20)) return AGG_ERR_INVALID_ARG;
    if (shard_bytes == 0 || shard_bytes % 16 != 0) return AGG_ERR_MISALIGNED;
    agg_ctx* c = new (std::nothrow) agg_ctx();
    if (!c) return AGG_ERR_NOMEM;
    c->W = world_size;
    c->rank = rank;
    c->shard_bytes = shard_bytes;
    c->n_signals = n_signals;
    c->epoch = 1;
    c->wait_limit_us = 2000000;
    c->tile_config = -1;
    c->rs_chunks = 1;
    c->rs_own_last = 1;
    int rc = AGG_OK;
    hipDeviceProp_t prop;
    int khz = 0;
    const size_t sig_bytes = (size_t)n_signals * kSignalStride * sizeof(int);
    const size_t ctr_bytes = ((size_t)n_signals + kMaxWorld * kMaxRsChunks + 32) * sizeof(int);   // producer counters, then one per chunk of a GEMM-RS slice
    if ((rc = hip_fail(hipGetDevice(&c->device))) != AGG_OK) goto fail;
    if ((rc = hip_fail(hipGetDeviceProperties(&prop, c->device))) != AGG_OK) goto fail;
    if ((rc = hip_fail(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, c->device))) != AGG_OK) goto fail;
    c->num_cus = prop.multiProcessorCount;
    c->wall_khz = khz > 0 ? khz : 100000;
    {
        int can = 0;
        if (hipDeviceGetAttribute(&can, hipDeviceAttributeCanUseStreamWaitValue, c->device) != hipSuccess) (void)hipGetLastError();
        c->can_wait_value = can;
    }
    if ((rc = hip_fail(hipMalloc((void**)&c->staging, (size_t)world_size * shard_bytes))) != AGG_OK) goto fail;
    if ((rc = hip_fail(hipMalloc((void**)&c->signals, sig_bytes))) != AGG_OK) goto fail;
    if ((rc = hip_fail(hipMalloc((void**)&c->counters, ctr_bytes))) != AGG_OK) goto fail;
    if ((rc = hip_fail(hipMalloc((void**)&c->err, 2048))) != AGG_OK) goto fail;
    if ((rc = hip_fail(hipMalloc((void**)&c->epoch_word, 256))) != AGG_OK) goto fail;
    if ((rc = hip_fail(hipMemset(c->signals, 0, sig_bytes))) != AGG_OK) goto fail;
    if ((rc = hip_fail(hipMemset(c->counters, 0, ctr_bytes))) != AGG_OK) goto fail;
    if ((rc = hip_fail(hipMemset(c->err, 0, 2048))) != AGG_OK) goto fail;
    if ((rc = hip_fail(hipMemset(c->epoch_word, 0, 256))) != AGG_OK) goto fail;
    if ((rc = hip_fail(hipStreamCreateWithFlags(&c->consumer_stream, hipStreamNonBlocking))) != AGG_OK) goto fail;
    if ((rc = pick_concurrent_stream(c)) != AGG_OK) goto fail;
    if ((rc = hip_fail(hipEventCreateWithFlags(&c->gemm_done, hipEventDisableTiming))) != AGG_OK) goto fail;
    if ((rc = hip_fail(hipEventCreateWithFlags(&c->b_nk_free, hipEventDisableTiming))) != AGG_OK) goto fail;
    if ((rc = hip_fail(hipGetSymbolAddress((void**)&c->static_scratch, HIP_SYMBOL(scratch)))) != AGG_OK) goto fail;
    if ((rc = hip_fail(hipDeviceSynchronize())) != AGG_OK) goto fail;
    *out = c;
    return AGG_OK;
fail:
    symm_free(c);
    return rc;
}

int symm_free(agg_ctx* c)
{
    if (!c) return AGG_ERR_INVALID_ARG;
    (void)hipDeviceSynchronize();
    if (c->producer_stream) (void)hipStreamDestroy(c->producer_stream);
    if (c->consumer_stream) (void)hipStreamDestroy(c->consumer_stream);
    if (c->gemm_done) (void)hipEventDestroy(c->gemm_done);
    if (c->b_nk_free) (void)hipEventDestroy(c->b_nk_free);
    if (c->b_nk) (void)hipFree(c->b_nk);
    if (c->moe_ws) (void)hipFree(c->moe_ws);
    if (c->moe_tab) (void)hipFree(c->moe_tab);
    if (c->staging) (void)hipFree(c->staging);
    if (c->signals) (void)hipFree(c->signals);
    if (c->counters) (void)hipFree(c->counters);
    if (c->err) (void)hipFree(c->err);
    if (c->epoch_word) (void)hipFree(c->epoch_word);
    (void)hipGetLastError();
    delete c;
    return AGG_OK;
}

void* symm_staging(agg_ctx* c) { return c ? c->staging : nullptr; }
int32_t* symm_signals(agg_ctx* c) { return c ? c->signals : nullptr; }
int symm_epoch(agg_ctx* c) { return c ? c->epoch : AGG_ERR_INVALID_ARG; }

int symm_streams(agg_ctx* c, void** producer_stream, void** consumer_stream)
{
    if (!c || !producer_stream || !consumer_stream) return AGG_ERR_INVALID_ARG;
    *producer_stream = (void*)c->producer_stream;
    *consumer_stream = (void*)c->consumer_stream;
    return AGG_OK;
}

int signal_reset(agg_ctx* c, void* stream)
{
    if (!c) return AGG_ERR_INVALID_ARG;
    if (c->epoch >= 0x7ffffff0) return AGG_ERR_INVALID_ARG;   // 2^31 runs: allocate a new context
    // with the epoch kept on the device, the reset is a one-thread kernel on the caller's stream (a HIP graph can
    // record it, and every replay advances the epoch); the host's count of resets is kept as well
    if (c->device_epoch) {
        const int rc = hip_fail(launch_epoch_advance(c->epoch_word, (hipStream_t)stream));
        if (rc != AGG_OK) return rc;
    }
    c->epoch += 1;
    return AGG_OK;
}

int agg_set_device_epoch(agg_ctx* c, int on)
{
    if (!c || (on != 0 && on != 1)) return AGG_ERR_INVALID_ARG;
    // both directions start from a quiet device: the word and the host's count are made equal
    HIP_TRY(hipDeviceSynchronize());
    if (on) {
        HIP_TRY(hipMemcpy(c->epoch_word, &c->epoch, sizeof(int), hipMemcpyHostToDevice));
    } else if (c->device_epoch) {
        int e = 0;
        HIP_TRY(hipMemcpy(&e, c->epoch_word, sizeof(int), hipMemcpyDeviceToHost));
        if (e > c->epoch) c->epoch = e;       // replays of a graph advanced the device's count past the host's
    }
    c->device_epoch = on;
    return AGG_OK;
}

int signal_set(agg_ctx* c, int index, void* stream)
{
    if (!c || index < 0 || index >= c->n_signals) return AGG_ERR_INVALID_ARG;
    return hip_fail(launch_signal_set(c->signals + (size_t)index * kSignalStride, c->epoch,
                                      c->device_epoch ? c->epoch_word : nullptr, (hipStream_t)stream));
}

int agg_set_wait_limit_us(agg_ctx* c, uint64_t us)
{
    if (!c || us == 0 || us > 600ull * 1000 * 1000) return AGG_ERR_INVALID_ARG;
    c->wait_limit_us = us;
    return AGG_OK;
}

int agg_set_local_shard(agg_ctx* c, const void* local_shard)
{
    if (!c) return AGG_ERR_INVALID_ARG;
    if (local_shard && !aligned16(local_shard)) return AGG_ERR_MISALIGNED;
    c->local_shard = local_shard;
    return AGG_OK;
}

int agg_set_tile_order(agg_ctx* c, int order)
{
    if (!c || (order != AGG_ORDER_ROTATED && order != AGG_ORDER_SUBCHUNK)) return AGG_ERR_INVALID_ARG;
    c->tile_order = order;
    return AGG_OK;
}

int agg_set_rs_chunks(agg_ctx* c, int chunks)
{
    if (!c || chunks < 1 || chunks > kMaxRsChunks || chunks > c->n_signals / c->W) return AGG_ERR_INVALID_ARG;
    c->rs_chunks = chunks;
    return AGG_OK;
}

int agg_set_rs_own_slice_last(agg_ctx* c, int on)
{
    if (!c || (on != 0 && on != 1)) return AGG_ERR_INVALID_ARG;
    c->rs_own_last = on;
    return AGG_OK;
}

int agg_set_link_rate(agg_ctx* c, double gigabytes_per_second)
{
    if (!c || !(gigabytes_per_second >= 0.0) || gigabytes_per_second > 1e6) return AGG_ERR_INVALID_ARG;
    c->link_GBps = gigabytes_per_second;
    return AGG_OK;
}

int agg_set_tile_config(agg_ctx* c, int cfg)
{
    if (!c || cfg < -1 || cfg >= TILE_CONFIGS) return AGG_ERR_INVALID_ARG;
    c->tile_config = cfg;
    return AGG_OK;
}

int agg_status(agg_ctx* c)
{
    if (!c) return AGG_ERR_INVALID_ARG;
    HIP_TRY(hipDeviceSynchronize());
    int h = 0;
    HIP_TRY(hipMemcpy(&h, c->err, sizeof h, hipMemcpyDeviceToHost));
    if (h != 0) {
        HIP_TRY(hipMemset(c->err, 0, sizeof h));
        HIP_TRY(hipDeviceSynchronize());
        return AGG_ERR_TIMEOUT;
    }
    return AGG_OK;
}

int agg_reserve_b_kn(agg_ctx* c, int N, int K)
{
    if (!c || N < 0 || K < 0) return AGG_ERR_INVALID_ARG;
    const size_t need = (size_t)N * K;
    if (c->b_nk_elems >= need) return AGG_OK;
    HIP_TRY(hipDeviceSynchronize());
    if (c->b_nk) (void)hipFree(c->b_nk);
    c->b_nk = nullptr;
    c->b_nk_elems = 0;
    HIP_TRY(hipMalloc((void**)&c->b_nk, need * sizeof(uint16_t)));
    c->b_nk_elems = need;
    return AGG_OK;
}

int agg_reserve_moe(agg_ctx* c, int Ttok, int topk, int E, int N)
{
    if (!c || Ttok < 0 || topk < 1 || E < 1 || E > 4096 || N < 0) return AGG_ERR_INVALID_ARG;
    const long long cap = moe_table_bound((long long)Ttok * topk, E, N);
    if (cap > (1ll << 28)) return AGG_ERR_UNSUPPORTED_SHAPE;
    if (!c->moe_ws) {
        HIP_TRY(hipDeviceSynchronize());
        HIP_TRY(hipMalloc((void**)&c->moe_ws, kMoeCtrlBytes));
        HIP_TRY(hipMemset(c->moe_ws, 0, kMoeCtrlBytes));         // the routing's counters start at zero
    }
    if (c->moe_tab_cap < cap) {
        HIP_TRY(hipDeviceSynchronize());
        if (c->moe_tab) (void)hipFree(c->moe_tab);
        c->moe_tab = nullptr;
        c->moe_tab_cap = 0;
        HIP_TRY(hipMalloc((void**)&c->moe_tab, (size_t)cap * sizeof(MoeTile)));
        c->moe_tab_cap = (int)cap;
    }
    return AGG_OK;
}

int ag_producer_emulate(agg_ctx* c, const void* const* remote_shards, const int* arrival_order, int n_arrivals,
                        int mode, int n_workgroups, void* producer_stream)
{
    if (!c || !remote_shards) return AGG_ERR_INVALID_ARG;
    const bool skip_local = (mode & AGG_PRODUCER_SKIP_LOCAL) != 0;
    const bool local_last = (mode & AGG_PRODUCER_LOCAL_LAST) != 0 && !skip_local;
    const int threads = (mode & AGG_PRODUCER_NARROW) ? 64 : 256;
    mode &= ~(AGG_PRODUCER_SKIP_LOCAL | AGG_PRODUCER_LOCAL_LAST | AGG_PRODUCER_NARROW);
    if (mode != AGG_PRODUCER_KERNEL && mode != AGG_PRODUCER_SDMA && mode != AGG_PRODUCER_LINKS) return AGG_ERR_INVALID_ARG;
    if (n_workgroups < 0 || n_workgroups > 4096) return AGG_ERR_INVALID_ARG;
    const int W = c->W;
    if (arrival_order && (n_arrivals < 0 || n_arrivals > W - 1)) return AGG_ERR_INVALID_ARG;
    const int cps = c->n_signals / W;
    if (c->shard_bytes % ((size_t)cps * 16) != 0) return AGG_ERR_MISALIGNED;
    ProducerArgs a{};
    bool used[kMaxWorld] = {false};
    a.n_jobs = 0;
    if (!skip_local && !local_last) a.rank_of[a.n_jobs++] = c->rank;   // the local copy comes first (Algorithm 2)
    used[c->rank] = true;
    const int n = arrival_order ? n_arrivals : W - 1;
    for (int j = 0; j < n; ++j) {
        const int r = arrival_order ? arrival_order[j] : (c->rank + 1 + j) % W;
        if (r < 0 || r >= W || used[r]) return AGG_ERR_INVALID_ARG;
        used[r] = true;
        a.rank_of[a.n_jobs++] = r;
    }
    if (local_last) a.rank_of[a.n_jobs++] = c->rank;   // ... or last, for a consumer that reads its own shard in place
    for (int j = 0; j < a.n_jobs; ++j) {
        a.src[j] = remote_shards[a.rank_of[j]];
        if (!a.src[j]) return AGG_ERR_INVALID_ARG;
        if (!aligned16(a.src[j])) return AGG_ERR_MISALIGNED;
    }
    if (a.n_jobs == 0) return AGG_OK;
    a.T = c->staging;
    a.shard_bytes = (long long)c->shard_bytes;
    a.chunks_per_shard = cps;
    a.chunk_bytes = (long long)(c->shard_bytes / cps);
    a.flags = c->signals;
    a.counters = c->counters;
    a.epoch = c->epoch;
    a.epoch_ptr = c->device_epoch ? c->epoch_word : nullptr;
    hipStream_t st = (hipStream_t)producer_stream;
    // a workgroup addresses its part of a chunk with 32-bit offsets
    if (mode != AGG_PRODUCER_SDMA) {
        const int nwg_ = n_workgroups > 0 ? n_workgroups : (c->producer_wgs > 0 ? c->producer_wgs : c->num_cus);
        const long long sharers = mode == AGG_PRODUCER_LINKS ? (nwg_ / (a.n_jobs > 0 ? a.n_jobs : 1) > 0 ? nwg_ / a.n_jobs : 1)
                                                             : (a.chunk_bytes / 65536 < nwg_ ? (a.chunk_bytes / 65536 > 0 ? a.chunk_bytes / 65536 : 1) : nwg_);
        if (a.chunk_bytes / sharers >= (1ll << 31) - 65536) return AGG_ERR_UNSUPPORTED_SHAPE;
    }
    if (mode == AGG_PRODUCER_KERNEL) {
        const int nwg = n_workgroups > 0 ? n_workgroups : (c->producer_wgs > 0 ? c->producer_wgs : c->num_cus);
        if (threads == 64 && a.n_jobs >= 2 && a.rank_of[0] != c->rank) {
            // Narrow copy, consumer reading its own shard in place: the local shard's tiles occupy only some of the
            // consumer's workgroups, and the others start on the first shard to arrive -- all of it, in the first round
            // of tiles.  That shard is therefore copied at full width (it lands in half the time), the rest by
            // one-wave workgroups.
            ProducerArgs first = a;
            first.n_jobs = 1;
            int rc = hip_fail(launch_producer(first, nwg, 256, st));
            if (rc != AGG_OK) return rc;
            ProducerArgs rest = a;
            rest.n_jobs = a.n_jobs - 1;
            for (int j = 0; j < rest.n_jobs; ++j) {
                rest.src[j] = a.src[j + 1];
                rest.rank_of[j] = a.rank_of[j + 1];
            }
            return hip_fail(launch_producer(rest, nwg, threads, st));
        }
        return hip_fail(launch_producer(a, nwg, threads, st));
    }
    if (mode == AGG_PRODUCER_LINKS) {
        // the local copy first, at full width (it crosses no link); then every peer on a link of its own
        const int nwg = n_workgroups > 0 ? n_workgroups : (c->producer_wgs > 0 ? c->producer_wgs : c->num_cus);
        const bool has_local = !skip_local;
        const int first_remote = (has_local && !local_last) ? 1 : 0;
        const int local_job = local_last ? a.n_jobs - 1 : 0;
        if (has_local && !local_last) {
            ProducerArgs loc = a;
            loc.n_jobs = 1;
            int rc = hip_fail(launch_producer(loc, nwg, threads, st));
            if (rc != AGG_OK) return rc;
        }
        ProducerArgs rem = a;
        rem.n_jobs = a.n_jobs - (has_local ? 1 : 0);
        for (int j = 0; j < rem.n_jobs; ++j) {
            rem.src[j] = a.src[j + first_remote];
            rem.rank_of[j] = a.rank_of[j + first_remote];
        }
        // wall-clock ticks per byte of one link
        rem.ticks_per_byte = c->link_GBps > 0.0 ? ((double)c->wall_khz * 1e3) / (c->link_GBps * 1e9) : 0.0;
        int rc = hip_fail(launch_producer_links(rem, nwg, st));
        if (rc != AGG_OK || !(has_local && local_last)) return rc;
        ProducerArgs loc = a;
        loc.n_jobs = 1;
        loc.src[0] = a.src[local_job];
        loc.rank_of[0] = a.rank_of[local_job];
        return hip_fail(launch_producer(loc, nwg, threads, st));
    }
    // copy engine: one transfer per chunk, then a second, tiny transfer that carries only the signal (Section 3.6)
    if (!c->device_epoch) HIP_TRY(launch_signal_set(c->epoch_word, c->epoch, nullptr, st));   // else the word is the epoch already
    for (int j = 0; j < a.n_jobs; ++j) {
        const int r = a.rank_of[j];
        for (int ch = 0; ch < cps; ++ch) {
            const size_t off = (size_t)ch * a.chunk_bytes;
            HIP_TRY(hipMemcpyAsync(c->staging + (size_t)r * c->shard_bytes + off, (const char*)a.src[j] + off,
                                   (size_t)a.chunk_bytes, hipMemcpyDeviceToDeviceNoCU, st));
            HIP_TRY(hipMemcpyAsync(c->signals + (size_t)(r * cps + ch) * kSignalStride, c->epoch_word, sizeof(int),
                                   hipMemcpyDeviceToDeviceNoCU, st));
        }
    }
    return AGG_OK;
}

int ag_gemm(agg_ctx* c, int M, int N, int K, const void* B, int ldb, int b_layout, void* C, int ldc, int c_dtype,
            void* consumer_stream)
{
    if (!c) return AGG_ERR_INVALID_ARG;
    int rc = check_gemm_operands(M, N, K, B, ldb, b_layout, C, ldc, c_dtype);
    if (rc != AGG_OK) return rc;
    if (M % c->W != 0) return AGG_ERR_UNSUPPORTED_SHAPE;
    if (M == 0 || N == 0) return AGG_OK;
    const int Ms = M / c->W;
    if ((size_t)Ms * K * 2 != c->shard_bytes) return AGG_ERR_UNSUPPORTED_SHAPE;
    const int cps = c->n_signals / c->W;
    if (Ms % cps != 0) return AGG_ERR_UNSUPPORTED_SHAPE;
    GemmParams p{};
    p.A = (const uint16_t*)c->staging;
    p.A_local = (const uint16_t*)c->local_shard;
    p.local_lo = c->rank * Ms;
    p.local_hi = p.local_lo + Ms;
    if ((rc = resolve_b(c, B, ldb, b_layout, N, K, (hipStream_t)consumer_stream, &p.B, &p.ldb)) != AGG_OK) return rc;
    p.C = C;
    p.lda = K;
    p.ldc = ldc;
    p.M = M;
    p.N = N;
    p.K = K;
    p.c_is_f32 = c_dtype == AGG_F32;
    p.c_vec_ok = aligned16(C) && ((long long)ldc * (p.c_is_f32 ? 4 : 2)) % 16 == 0;
    const int cfg = choose_tile(c, M, N);
    fill_schedule(p, cfg, Ms, c->rank * Ms);
    {
        // sub-chunk order (Section 3.7, full mesh): possible when shards and chunks are whole numbers of tiles
        const TileShape t = tile_shape(cfg);
        const int rows_per_chunk = Ms / cps;
        if (c->tile_order == AGG_ORDER_SUBCHUNK && Ms % t.bm == 0 && rows_per_chunk % t.bm == 0) {
            p.order = AGG_ORDER_SUBCHUNK;
            p.tiles_per_shard = Ms / t.bm;
            p.tiles_per_chunk = rows_per_chunk / t.bm;
            p.world = c->W;
            p.rank = c->rank;
        }
    }
    p.flags = c->signals;
    p.epoch = c->epoch;
    p.epoch_ptr = c->device_epoch ? c->epoch_word : nullptr;
    p.rows_per_flag = Ms / cps;
    p.n_flags = c->n_signals;
    p.wait_ticks = wait_ticks(c);
    p.err = c->err;
    const long long tiles = (long long)p.tiles_m * p.tiles_n;
    const int grid = (int)(tiles < c->num_cus ? tiles : c->num_cus);
    if ((rc = hip_fail(launch_gemm(p, cfg, grid, (hipStream_t)consumer_stream))) != AGG_OK) return rc;
    return b_kn_launched(c, b_layout, (hipStream_t)consumer_stream);
}

static int reduce_impl(agg_ctx* c, int Ms, int N, const float* const* slots, void* R, int ldr, int r_dtype, int n_workgroups,
                       void* stream, bool beside_gemm)
{
    if (!c || !slots || Ms < 0 || N < 0 || n_workgroups < 0 || n_workgroups > 65536) return AGG_ERR_INVALID_ARG;
    if (r_dtype != AGG_BF16 && r_dtype != AGG_F32) return AGG_ERR_INVALID_ARG;
    if (Ms == 0 || N == 0) return AGG_OK;
    if (!R || ldr < N) return AGG_ERR_INVALID_ARG;
    const long long n = (long long)Ms * N;
    if (n % 4 != 0) return AGG_ERR_UNSUPPORTED_SHAPE;
    if (ldr != N && (N % 4 != 0)) return AGG_ERR_UNSUPPORTED_SHAPE;
    const int esz = r_dtype == AGG_F32 ? 4 : 2;
    if (reinterpret_cast<uintptr_t>(R) % (4 * esz) != 0 || (ldr != N && ldr % 4 != 0)) return AGG_ERR_MISALIGNED;
    ReduceArgs a{};
    a.W = c->W;
    for (int w = 0; w < c->W; ++w) {
        if (!slots[w]) return AGG_ERR_INVALID_ARG;
        if (!aligned16(slots[w])) return AGG_ERR_MISALIGNED;
        a.slot[w] = slots[w];
    }
    a.n_vec4 = n / 4;
    a.row_vec4 = (ldr != N) ? N / 4 : 0;
    a.R = R;
    a.ldr = ldr;
    a.r_is_f32 = r_dtype == AGG_F32;
    a.N = N;
    a.flags = c->signals;
    a.flag_step = c->n_signals / c->W;
    a.chunks = c->rs_chunks;
    if (a.chunks > 1) {
        if (Ms % a.chunks != 0 || ((long long)(Ms / a.chunks) * N) % 4 != 0) return AGG_ERR_UNSUPPORTED_SHAPE;
        a.chunk_vec4 = (long long)(Ms / a.chunks) * N / 4;
    }
    a.epoch = c->epoch;
    a.epoch_ptr = c->device_epoch ? c->epoch_word : nullptr;
    a.wait_ticks = wait_ticks(c);
    a.err = c->err;
    int nwg = n_workgroups;
    if (nwg == 0) {
        // persistent: three workgroups per two CUs, each walking many blocks (one acquire per workgroup, not per
        // block).  Measured: 6.2 TB/s; one per CU reaches 6.27 alone but 5.8 when the placement of the workgroups
        // is less than perfect (as found inside longer runs); two per CU 6.1, three 5.3.
        const long long need = (a.n_vec4 + 255) / 256;
        // Beside the GEMM a CU has room for one reducer workgroup only (one 64-register wave per SIMD).
        const long long want = beside_gemm ? (long long)c->num_cus : (long long)c->num_cus * 3 / 2;
        nwg = (int)(need < want ? need : want);
        if (nwg < 1) nwg = 1;
    }
    return hip_fail(launch_reduce(a, nwg, (hipStream_t)stream, beside_gemm));
}

int rs_reduce(agg_ctx* c, int Ms, int N, const float* const* slots, void* R, int ldr, int r_dtype, int n_workgroups,
              void* stream)
{
    return reduce_impl(c, Ms, N, slots, R, ldr, r_dtype, n_workgroups, stream, false);
}

// Tuning in the manner of Section 3.8: the unit that is timed is the whole overlapped function -- reset of the
// signals, arrival on the producer stream, gated GEMM on the consumer stream, join -- never a kernel on its own, whose
// waits would find the signals of the previous run.  One candidate configuration per run of the function.
int agg_autotune_ag_gemm(agg_ctx* c, int M, int N, int K, const void* B, int ldb, int b_layout, void* C, int ldc,
                         int c_dtype, const void* const* remote_shards, int producer_mode, int runs_per_config,
                         agg_tune_result* out)
{
    if (!c || !out || runs_per_config < 1 || runs_per_config > 1000) return AGG_ERR_INVALID_ARG;
    const int saved_tile = c->tile_config, saved_order = c->tile_order, saved_wgs = c->producer_wgs;
    const int tiles[4] = {TILE_256x224 | TILE_K32, TILE_256x256 | TILE_K32, TILE_128x256 | TILE_K32, TILE_128x128 | TILE_K32};
    const int orders[2] = {AGG_ORDER_ROTATED, AGG_ORDER_SUBCHUNK};
    const int wgs[3] = {c->num_cus / 2 > 0 ? c->num_cus / 2 : 1, c->num_cus, 2 * c->num_cus};
    hipEvent_t e0 = nullptr, e1 = nullptr, join = nullptr;
    int rc = AGG_OK;
    float best = 1e30f;
    agg_tune_result res{};
    if ((rc = hip_fail(hipEventCreate(&e0))) != AGG_OK) return rc;
    if ((rc = hip_fail(hipEventCreate(&e1))) != AGG_OK) { (void)hipEventDestroy(e0); return rc; }
    if ((rc = hip_fail(hipEventCreateWithFlags(&join, hipEventDisableTiming))) != AGG_OK) {
        (void)hipEventDestroy(e0); (void)hipEventDestroy(e1); return rc;
    }
    const bool sdma = (producer_mode & 0xff) == AGG_PRODUCER_SDMA;
    for (int ti = 0; ti < 4 && rc == AGG_OK; ++ti)
        for (int oi = 0; oi < 2 && rc == AGG_OK; ++oi)
            for (int wi = 0; wi < (sdma ? 1 : 3) && rc == AGG_OK; ++wi) {
                c->tile_config = tiles[ti];
                c->tile_order = orders[oi];
                c->producer_wgs = wgs[wi];
                std::vector<float> times;
                // untimed runs first: one per candidate, and a longer series before the very first candidate, so
                // that the chip's clocks have settled under load before anything is compared
                const int warm = res.configs_tried == 0 ? 30 : 1;
                for (int it = 0; it < runs_per_config + warm && rc == AGG_OK; ++it) {
                    if ((rc = signal_reset(c, c->consumer_stream)) != AGG_OK) break;   // ahead of the fork below
                    // fork: both streams start from the same point
                    if ((rc = hip_fail(hipEventRecord(e0, c->consumer_stream))) != AGG_OK) break;
                    if ((rc = hip_fail(hipStreamWaitEvent(c->producer_stream, e0, 0))) != AGG_OK) break;
                    if ((rc = ag_producer_emulate(c, remote_shards, nullptr, 0, producer_mode, 0, c->producer_stream)) != AGG_OK) break;
                    if ((rc = ag_gemm(c, M, N, K, B, ldb, b_layout, C, ldc, c_dtype, c->consumer_stream)) != AGG_OK) break;
                    // join: the function is over when both parts are
                    if ((rc = hip_fail(hipEventRecord(join, c->producer_stream))) != AGG_OK) break;
                    if ((rc = hip_fail(hipStreamWaitEvent(c->consumer_stream, join, 0))) != AGG_OK) break;
                    if ((rc = hip_fail(hipEventRecord(e1, c->consumer_stream))) != AGG_OK) break;
                    if ((rc = hip_fail(hipEventSynchronize(e1))) != AGG_OK) break;
                    float ms = 0.f;
                    if ((rc = hip_fail(hipEventElapsedTime(&ms, e0, e1))) != AGG_OK) break;
                    if (it >= warm) times.push_back(ms);
                }
                float best_here = 1e30f;
                if (!times.empty()) {
                    std::sort(times.begin(), times.end());
                    best_here = times[times.size() / 2];       // the median run
                }
                if (rc == AGG_OK) rc = agg_status(c);          // a candidate whose waits time out is an error, not a result
                ++res.configs_tried;
                if (rc == AGG_OK && best_here < best) {
                    best = best_here;
                    res.tile_config = tiles[ti];
                    res.tile_order = orders[oi];
                    res.producer_workgroups = sdma ? 0 : wgs[wi];
                    res.best_ms = best_here;
                }
            }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    (void)hipEventDestroy(join);
    if (rc != AGG_OK) {
        c->tile_config = saved_tile;
        c->tile_order = saved_order;
        c->producer_wgs = saved_wgs;
        return rc;
    }
    c->tile_config = res.tile_config;
    c->tile_order = res.tile_order;
    c->producer_wgs = res.producer_workgroups;
    tune_table_put(c->W, M, N, K, res);
    *out = res;
    return AGG_OK;
}

int gemm_rs_scatter(agg_ctx* c, int M, int N, int Kl, const void* A_local, int lda, const void* B_local, int ldb,
                    int b_layout, float* const* slice_dst, float* P_other, int32_t* const* slice_signal,
                    int first_slice, void* gemm_stream)
{
    if (!c || !slice_dst) return AGG_ERR_INVALID_ARG;
    if (M % c->W != 0) return AGG_ERR_UNSUPPORTED_SHAPE;
    if (first_slice < 0 || first_slice >= c->W) return AGG_ERR_INVALID_ARG;
    const int W = c->W, Ms = M / W;
    if (M == 0 || N == 0) return AGG_OK;
    if (Ms % c->rs_chunks != 0) return AGG_ERR_UNSUPPORTED_SHAPE;
    // every slice needs somewhere to go
    const void* any_dst = P_other;
    for (int w = 0; w < W; ++w) {
        if (!slice_dst[w] && !P_other) return AGG_ERR_INVALID_ARG;
        if (slice_dst[w] && !aligned16(slice_dst[w])) return AGG_ERR_MISALIGNED;
        if (slice_signal && slice_signal[w] && reinterpret_cast<uintptr_t>(slice_signal[w]) % 4 != 0) return AGG_ERR_MISALIGNED;
        if (!any_dst) any_dst = slice_dst[w];
    }
    int rc = check_gemm_operands(M, N, Kl, B_local, ldb, b_layout, any_dst, N, AGG_F32);
    if (rc != AGG_OK) return rc;
    if (!A_local || lda < Kl) return AGG_ERR_INVALID_ARG;
    if (lda % 8 != 0 || !aligned16(A_local)) return AGG_ERR_MISALIGNED;
    if (P_other && !aligned16(P_other)) return AGG_ERR_MISALIGNED;

    GemmParams p{};
    p.A = (const uint16_t*)A_local;
    if ((rc = resolve_b(c, B_local, ldb, b_layout, N, Kl, (hipStream_t)gemm_stream, &p.B, &p.ldb)) != AGG_OK) return rc;
    p.C = P_other;
    p.lda = lda;
    p.ldc = N;
    p.M = M;
    p.N = N;
    p.K = Kl;
    p.c_is_f32 = 1;
    p.c_vec_ok = N % 4 == 0;              // every destination is 16-byte aligned (checked above)
    p.epoch = c->epoch;
    p.epoch_ptr = c->device_epoch ? c->epoch_word : nullptr;
    p.err = c->err;
    p.wait_ticks = wait_ticks(c);
    p.n_slices = W;
    p.slice_rows = Ms;
    p.slice_chunks = c->rs_chunks;
    p.chunk_rows = Ms / c->rs_chunks;
    p.ldc_slice = N;
    p.slice_ctr = c->counters + c->n_signals;          // counters of their own, after the producer's
    for (int w = 0; w < W; ++w) {
        p.slice_dst[w] = slice_dst[w];
        p.slice_flag[w] = slice_signal ? slice_signal[w] : nullptr;
    }
    const int cfg = choose_tile(c, M, N);
    fill_schedule(p, cfg, Ms, first_slice * Ms);
    const long long tiles = (long long)p.tiles_m * p.tiles_n;
    const int grid = (int)(tiles < c->num_cus ? tiles : c->num_cus);
    if ((rc = hip_fail(launch_gemm(p, cfg, grid, (hipStream_t)gemm_stream))) != AGG_OK) return rc;
    return b_kn_launched(c, b_layout, (hipStream_t)gemm_stream);
}

int gemm_rs(agg_ctx* c, int M, int N, int Kl, const void* A_local, int lda, const void* B_local, int ldb, int b_layout,
            const float* const* slots, float* P_other, void* R, int ldr, int r_dtype, void* gemm_stream,
            void* reduce_stream)
{
    if (!c || !slots) return AGG_ERR_INVALID_ARG;
    if (M % c->W != 0) return AGG_ERR_UNSUPPORTED_SHAPE;
    const int W = c->W, Ms = M / W;
    if (M == 0 || N == 0) return AGG_OK;
    if (!slots[c->rank]) return AGG_ERR_INVALID_ARG;
    if (Ms % c->rs_chunks != 0 || ((long long)(Ms / c->rs_chunks) * N) % 4 != 0) return AGG_ERR_UNSUPPORTED_SHAPE;
    // validate the reduction's arguments before anything is enqueued
    if (!R || ldr < N || (r_dtype != AGG_BF16 && r_dtype != AGG_F32)) return AGG_ERR_INVALID_ARG;
    if (((long long)Ms * N) % 4 != 0 || (ldr != N && N % 4 != 0)) return AGG_ERR_UNSUPPORTED_SHAPE;
    for (int w = 0; w < W; ++w)
        if (!slots[w] || !aligned16(slots[w])) return slots[w] ? AGG_ERR_MISALIGNED : AGG_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(R) % (4 * (r_dtype == AGG_F32 ? 4 : 2)) != 0 || (ldr != N && ldr % 4 != 0))
        return AGG_ERR_MISALIGNED;

    int32_t* own_flag = c->signals + (size_t)c->rank * (c->n_signals / W) * kSignalStride;
    int rc;
    if (P_other) {
        // all M rows: the own slice first and straight into its slot, the others' rows into P_other
        float* dst[kMaxWorld] = {nullptr};
        int32_t* sig[kMaxWorld] = {nullptr};
        dst[c->rank] = const_cast<float*>(slots[c->rank]);
        sig[c->rank] = own_flag;
        const int first = c->rs_own_last ? (c->rank + 1) % W : c->rank;
        rc = gemm_rs_scatter(c, M, N, Kl, A_local, lda, B_local, ldb, b_layout, dst, P_other, sig, first, gemm_stream);
    } else {
        // only the own slice is wanted: a GEMM over its Ms rows, seen as a world of one slice
        rc = check_gemm_operands(Ms, N, Kl, B_local, ldb, b_layout, slots[c->rank], N, AGG_F32);
        if (rc != AGG_OK) return rc;
        if (!A_local || lda < Kl) return AGG_ERR_INVALID_ARG;
        if (lda % 8 != 0 || !aligned16(A_local)) return AGG_ERR_MISALIGNED;
        GemmParams p{};
        p.A = (const uint16_t*)A_local + (long long)c->rank * Ms * lda;
        if ((rc = resolve_b(c, B_local, ldb, b_layout, N, Kl, (hipStream_t)gemm_stream, &p.B, &p.ldb)) != AGG_OK) return rc;
        p.C = (void*)slots[c->rank];
        p.lda = lda;
        p.ldc = N;
        p.M = Ms;
        p.N = N;
        p.K = Kl;
        p.c_is_f32 = 1;
        p.c_vec_ok = N % 4 == 0;
        p.epoch = c->epoch;
        p.epoch_ptr = c->device_epoch ? c->epoch_word : nullptr;
        p.err = c->err;
        p.wait_ticks = wait_ticks(c);
        p.n_slices = 1;
        p.slice_rows = Ms;
        p.slice_chunks = c->rs_chunks;
        p.chunk_rows = Ms / c->rs_chunks;
        p.ldc_slice = N;
        p.slice_ctr = c->counters + c->n_signals;
        p.slice_flag[0] = own_flag;
        const int cfg = choose_tile(c, Ms, N);
        fill_schedule(p, cfg, Ms, 0);
        const long long tiles = (long long)p.tiles_m * p.tiles_n;
        const int grid = (int)(tiles < c->num_cus ? tiles : c->num_cus);
        rc = hip_fail(launch_gemm(p, cfg, grid, (hipStream_t)gemm_stream));
        if (rc == AGG_OK) rc = b_kn_launched(c, b_layout, (hipStream_t)gemm_stream);
    }
    if (rc != AGG_OK) return rc;
    // The reducer waits for this rank's own slot, which the GEMM above produces.  A reducer that spun for that
    // signal inside the kernel could hold the registers the GEMM's workgroups still need to become resident, and
    // the two would wait for each other; so the reduce stream itself waits (no compute unit is held) until the own
    // slice is signalled, and the reducer then runs beside the rest of the GEMM.  The stream wait ends at the
    // latest when the GEMM kernel has completed, so it needs no time limit of its own.
    // With the own slice computed last and cut into chunks, the stream waits for its first chunk only: by then every
    // workgroup of the (persistent) GEMM has long been resident, and the reducer takes the later chunks' signals itself.
    if (gemm_stream != reduce_stream) {
        bool waited = false;
        if (c->can_wait_value && !c->device_epoch) {   // (a stream wait compares with a value fixed at enqueue time)
            const int n_wait = (c->rs_own_last && P_other) ? 1 : c->rs_chunks;
            waited = true;
            for (int ch = 0; waited && ch < n_wait; ++ch)
                waited = hipStreamWaitValue32((hipStream_t)reduce_stream, own_flag + ch * kSignalStride, (uint32_t)c->epoch,
                                              hipStreamWaitValueGte, 0xFFFFFFFFu) == hipSuccess;
            if (!waited) (void)hipGetLastError();
        }
        if (!waited) {   // no stream wait on memory here: order the reducer after the whole GEMM
            if ((rc = hip_fail(hipEventRecord(c->gemm_done, (hipStream_t)gemm_stream))) != AGG_OK) return rc;
            if ((rc = hip_fail(hipStreamWaitEvent((hipStream_t)reduce_stream, c->gemm_done, 0))) != AGG_OK) return rc;
        }
    }
    return reduce_impl(c, Ms, N, slots, R, ldr, r_dtype, 0, reduce_stream, gemm_stream != reduce_stream);
}

// Routing + grouped GEMM, shared by ag_moe_gemm (A = T, rows gathered by token, tiles gated by the signals) and moe_rs
// (A = the routed rows themselves, nothing to wait for).
// The routing's control block (its first word is the tile count) and the tile table come from the caller of this
// function: the context's reserved buffers, or the library's static scratch.
// keep_lo < keep_hi: only the rows of tokens in [keep_lo, keep_hi) are wanted: the routing lists tiles for those rows only
// (one run of rows per expert, since tokens rise inside a segment).
static int grouped_gemm(agg_ctx* c, int Ttok, int topk, int E, int N, int K, const int32_t* topk_ids, const void* A,
                        bool gathered, const void* weights, int32_t* sorted_token, int32_t* seg_off, int32_t* pair_pos,
                        void* Y, int ldy, int y_dtype, hipStream_t stream, int* n_tiles_word, MoeTile* tab, long long tab_cap,
                        int keep_lo = 0, int keep_hi = 0)
{
    const long long P = (long long)Ttok * topk;
    const unsigned long long a_bytes = (unsigned long long)(gathered ? Ttok : P) * K * 2;
    if (P > (1ll << 30) || a_bytes >= (1ull << 31)) return AGG_ERR_UNSUPPORTED_SHAPE;   // 32-bit row offsets
    if (ldy < N) return AGG_ERR_INVALID_ARG;
    if (!aligned16(weights) || !aligned16(topk_ids) || !aligned16(A)) return AGG_ERR_MISALIGNED;
    if (reinterpret_cast<uintptr_t>(Y) % (y_dtype == AGG_F32 ? 4 : 2) != 0) return AGG_ERR_MISALIGNED;
    const int tpr = Ttok / c->W, cps = c->n_signals / c->W;

    // Tile shape: segments are ragged (about P / E rows each, a binomial spread around it).  Estimate the tiles
    // each shape would need with segments 15 % above the mean, in waves over the CUs, times the cost of a tile
    // (the small tile is bound by the global->LDS path: about 0.6 of the large tile's rate per flop).
    int cfg = c->tile_config;
    if (cfg < 0) {
        const int cand[3] = {TILE_256x224, TILE_256x256, TILE_128x128};
        const double eff[3] = {1.0, 1.0, 0.6};
        // (with a token range to keep, only the rows of those tokens get tiles)
        const double rows = 1.15 * (keep_lo < keep_hi ? (double)(keep_hi - keep_lo) * topk : (double)P) / E;
        double best = 1e300;
        for (int i = 0; i < 3; ++i) {
            const TileShape ts = tile_shape(cand[i]);
            const long long mt = (long long)((rows + ts.bm - 1) / ts.bm);
            const long long tiles = (long long)E * mt * ((N + ts.bn - 1) / ts.bn);
            const long long waves = (tiles + c->num_cus - 1) / c->num_cus;
            const double cost = (double)waves * ts.bm * ts.bn / eff[i];
            if (cost < best) { best = cost; cfg = cand[i]; }
        }
        cfg |= TILE_K32;
    }
    const TileShape t = tile_shape(cfg);
    const int tiles_n = (N + t.bn - 1) / t.bn;
    const long long cap = (P / t.bm + E) * tiles_n;              // sum over experts of ceil(rows / bm) <= P / bm + E
    if (cap > (1ll << 28)) return AGG_ERR_UNSUPPORTED_SHAPE;
    if (!n_tiles_word || !tab || tab_cap < cap) return AGG_ERR_NOT_RESERVED;
    MoeRouteArgs r{};
    r.topk_ids = topk_ids;
    r.P = (int)P;
    r.topk = topk;
    r.E = E;
    r.n_tiles_dev = n_tiles_word;
    r.seg_off = seg_off;
    r.sorted_token = sorted_token;
    r.pair_pos = pair_pos;
    r.keep_lo = keep_lo;
    r.keep_hi = keep_hi;
    r.bm = t.bm;
    r.tiles_n = tiles_n;
    r.rows_per_flag = gathered ? tpr / cps : 1;
    r.n_flags = c->n_signals;
    r.tile_tab = tab;
    r.tab_capacity = (int)cap;
    r.ctrl = (unsigned char*)n_tiles_word;
    r.wait_ticks = wait_ticks(c);
    r.err = c->err;
    int rc = hip_fail(launch_moe_route(r, stream));
    if (rc != AGG_OK) return rc;

    GemmParams p{};
    p.A = (const uint16_t*)A;
    p.B = (const uint16_t*)weights;
    p.C = Y;
    p.lda = K;
    p.ldb = K;
    p.ldc = ldy;
    p.M = (int)P;
    p.N = N;
    p.K = K;
    p.c_is_f32 = y_dtype == AGG_F32;
    p.c_vec_ok = aligned16(Y) && ((long long)ldy * (p.c_is_f32 ? 4 : 2)) % 16 == 0;
    p.tiles_n = tiles_n;
    p.flags = gathered ? c->signals : nullptr;
    p.epoch = c->epoch;
    p.epoch_ptr = c->device_epoch ? c->epoch_word : nullptr;
    p.n_flags = c->n_signals;
    p.rows_per_flag = r.rows_per_flag;
    p.wait_ticks = wait_ticks(c);
    p.err = c->err;
    p.row_index = gathered ? sorted_token : nullptr;      // nullptr: row p of the output reads row p of A
    p.tile_tab = tab;
    p.n_tiles_dev = r.n_tiles_dev;
    p.b_group_stride = (long long)N * K;
    p.a_bytes = (unsigned)a_bytes;
    const int grid = (int)(cap < c->num_cus ? cap : c->num_cus);
    return hip_fail(launch_gemm_grouped(p, cfg, grid, stream));
}

static int ag_moe_gemm_impl(agg_ctx* c, int Ttok, int topk, int E, int N, int K, const int32_t* topk_ids, const void* weights,
                            int32_t* sorted_token, int32_t* sorted_expert_offsets, void* Y, int ldy, int y_dtype, void* stream,
                            int* n_tiles_word, MoeTile* tab, long long tab_cap)
{
    if (!c || Ttok < 0 || topk < 1 || E < 1 || E > 4096 || N < 0 || K < 0) return AGG_ERR_INVALID_ARG;
    if (y_dtype != AGG_BF16 && y_dtype != AGG_F32) return AGG_ERR_INVALID_ARG;
    if (topk > E) return AGG_ERR_INVALID_ARG;
    if (Ttok == 0 || N == 0) return AGG_OK;
    if (!topk_ids || !weights || !sorted_token || !sorted_expert_offsets || !Y) return AGG_ERR_INVALID_ARG;
    if (K == 0 || K % 64 != 0 || K > (1 << 21)) return AGG_ERR_UNSUPPORTED_SHAPE;
    if (Ttok % c->W != 0) return AGG_ERR_UNSUPPORTED_SHAPE;
    const int tpr = Ttok / c->W;                                  // tokens per rank = rows per shard of T
    if ((size_t)tpr * K * 2 != c->shard_bytes) return AGG_ERR_UNSUPPORTED_SHAPE;
    const int cps = c->n_signals / c->W;
    if (tpr % cps != 0) return AGG_ERR_UNSUPPORTED_SHAPE;
    return grouped_gemm(c, Ttok, topk, E, N, K, topk_ids, c->staging, true, weights, sorted_token, sorted_expert_offsets,
                        nullptr, Y, ldy, y_dtype, (hipStream_t)stream, n_tiles_word, tab, tab_cap);
}

int ag_moe_gemm(agg_ctx* c, int Ttok, int topk, int E, int N, int K, const int32_t* topk_ids, const void* weights,
                int32_t* sorted_token, int32_t* sorted_expert_offsets, void* Y, int ldy, int y_dtype, void* stream)
{
    if (!c) return AGG_ERR_INVALID_ARG;
    return ag_moe_gemm_impl(c, Ttok, topk, E, N, K, topk_ids, weights, sorted_token, sorted_expert_offsets, Y, ldy, y_dtype,
                            stream, c->moe_ws, c->moe_tab, c->moe_tab_cap);
}

int ag_moe_gemm_static(agg_ctx* c, int Ttok, int topk, int E, int N, int K, const int32_t* topk_ids, const void* weights,
                       int32_t* sorted_token, int32_t* sorted_expert_offsets, void* Y, int ldy, int y_dtype, void* stream)
{
    if (!c || !c->static_scratch) return AGG_ERR_INVALID_ARG;
    // the table lives in the library's static device array: a problem whose table could exceed it is refused
    const long long room = (long long)((kStaticScratchBytes - kStaticTabOffset) / sizeof(MoeTile));
    if (Ttok > 0 && topk > 0 && E > 0 && N > 0 && moe_table_bound((long long)Ttok * topk, E, N) > room)
        return AGG_ERR_UNSUPPORTED_SHAPE;
    return ag_moe_gemm_impl(c, Ttok, topk, E, N, K, topk_ids, weights, sorted_token, sorted_expert_offsets, Y, ldy, y_dtype,
                            stream, (int*)c->static_scratch, (MoeTile*)(c->static_scratch + kStaticTabOffset), room);
}

int moe_rs(agg_ctx* c, int Ttok, int topk, int E, int N, int Kl, const void* H, const void* weights2,
           const int32_t* topk_ids, const float* gate, float* Y, int32_t* sorted_token, int32_t* sorted_expert_offsets,
           int32_t* pair_pos, const float* const* slots, float* Z_other, void* R, int ldr, int r_dtype,
           void* gemm_stream, void* reduce_stream)
{
    if (!c || Ttok < 0 || topk < 1 || topk > 64 || E < 1 || E > 4096 || N < 0 || Kl < 0 || !slots) return AGG_ERR_INVALID_ARG;
    if (topk > E) return AGG_ERR_INVALID_ARG;
    if (Ttok % c->W != 0) return AGG_ERR_UNSUPPORTED_SHAPE;
    if (Ttok == 0 || N == 0) return AGG_OK;
    if (!H || !weights2 || !topk_ids || !gate || !Y || !sorted_token || !sorted_expert_offsets || !pair_pos)
        return AGG_ERR_INVALID_ARG;
    if (Kl == 0 || Kl % 64 != 0 || Kl > (1 << 21) || N % 4 != 0) return AGG_ERR_UNSUPPORTED_SHAPE;
    const int W = c->W, Tr = Ttok / W;
    // the reduction's arguments, checked before anything is enqueued
    if (Tr % c->rs_chunks != 0) return AGG_ERR_UNSUPPORTED_SHAPE;      // (N % 4 == 0 makes every chunk whole float4s)
    if (!R || ldr < N || (r_dtype != AGG_BF16 && r_dtype != AGG_F32)) return AGG_ERR_INVALID_ARG;
    if (ldr != N && ldr % 4 != 0) return AGG_ERR_MISALIGNED;
    for (int w = 0; w < W; ++w)
        if (!slots[w] || !aligned16(slots[w])) return slots[w] ? AGG_ERR_MISALIGNED : AGG_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(R) % (4 * (r_dtype == AGG_F32 ? 4 : 2)) != 0) return AGG_ERR_MISALIGNED;
    if (!aligned16(Y) || !aligned16(gate) || (Z_other && !aligned16(Z_other))) return AGG_ERR_MISALIGNED;

    // 1. grouped GEMM on the routed rows (fp32 out)
    // Without Z_other only this rank's tokens are wanted: the GEMM then stores their rows of Y only and skips the tiles
    // that hold none of them (inside an expert's segment the tokens rise, so the rows of one rank are one run)
    const int keep_lo = Z_other ? 0 : c->rank * Tr, keep_hi = Z_other ? 0 : keep_lo + Tr;
    int rc = grouped_gemm(c, Ttok, topk, E, N, Kl, topk_ids, H, false, weights2, sorted_token, sorted_expert_offsets,
                          pair_pos, Y, N, AGG_F32, (hipStream_t)gemm_stream, c->moe_ws, c->moe_tab, c->moe_tab_cap,
                          keep_lo, keep_hi);
    if (rc != AGG_OK) return rc;
    // 2. top-k reduction: this rank's tokens into its own slot (first), the others' into Z_other
    TopkReduceArgs t{};
    t.Y = Y;
    t.pair_pos = pair_pos;
    t.gate = gate;
    t.T = Ttok;
    t.topk = topk;
    t.N = N;
    t.own_lo = c->rank * Tr;
    t.own_hi = t.own_lo + Tr;
    t.Z_own = const_cast<float*>(slots[c->rank]);
    t.Z_other = Z_other;
    if ((rc = hip_fail(launch_topk_reduce(t, c->num_cus * 4, (hipStream_t)gemm_stream))) != AGG_OK) return rc;
    // 3. notify: the own slot is complete; then the reducer, which waits for the peers' signals itself
    int32_t* own_flag = c->signals + (size_t)c->rank * (c->n_signals / W) * kSignalStride;
    for (int ch = 0; ch < c->rs_chunks; ++ch)   // the reduction above completes all row chunks of the slot at once
        if ((rc = hip_fail(launch_signal_set(own_flag + ch * kSignalStride, c->epoch, c->device_epoch ? c->epoch_word : nullptr,
                                             (hipStream_t)gemm_stream))) != AGG_OK)
            return rc;
    if (gemm_stream != reduce_stream) {
        bool waited = false;
        if (c->can_wait_value && !c->device_epoch) {   // (a stream wait compares with a value fixed at enqueue time)
            // with a chunked own slot: every chunk's signal, one after the other
            waited = true;
            for (int ch = 0; waited && ch < c->rs_chunks; ++ch)
                waited = hipStreamWaitValue32((hipStream_t)reduce_stream, own_flag + ch * kSignalStride, (uint32_t)c->epoch,
                                              hipStreamWaitValueGte, 0xFFFFFFFFu) == hipSuccess;
            if (!waited) (void)hipGetLastError();
        }
        if (!waited) {
            if ((rc = hip_fail(hipEventRecord(c->gemm_done, (hipStream_t)gemm_stream))) != AGG_OK) return rc;
            if ((rc = hip_fail(hipStreamWaitEvent((hipStream_t)reduce_stream, c->gemm_done, 0))) != AGG_OK) return rc;
        }
    }
    return rs_reduce(c, Tr, N, slots, R, ldr, r_dtype, 0, reduce_stream);
}

int agg_mfma_ceiling(agg_ctx* c, int iterations, int constant_operands, double* flop, void* stream)
{
    if (!c || iterations < 1 || iterations > (1 << 24) || !flop) return AGG_ERR_INVALID_ARG;
    // one workgroup of four waves per compute unit, 56 MFMAs of 16x16x32 per wave and iteration
    *flop = (double)c->num_cus * 4.0 * (double)iterations * 56.0 * (2.0 * 16 * 16 * 32);
    return hip_fail(launch_mfma_ceiling((float*)(c->err + 48), c->num_cus, iterations, constant_operands != 0,
                                        (hipStream_t)stream));
}

const char* agg_strerror(int code)
{
    switch (code) {
        case AGG_OK: return "ok";
        case AGG_ERR_INVALID_ARG: return "invalid argument";
        case AGG_ERR_UNSUPPORTED_SHAPE: return "unsupported shape or layout";
        case AGG_ERR_MISALIGNED: return "misaligned pointer or leading dimension";
        case AGG_ERR_HIP: return "HIP runtime error";
        case AGG_ERR_TIMEOUT: return "a kernel gave up waiting for a signal";
        case AGG_ERR_NOMEM: return "out of memory";
        case AGG_ERR_NOT_FOUND: return "no such entry";
        case AGG_ERR_IO: return "file could not be read or written";
        case AGG_ERR_NOT_RESERVED: return "workspace not reserved (agg_reserve_b_kn / agg_reserve_moe) or too small";
        default: return "unknown error";
    }
}

int agg_device_info(int* compute_units, int* clock_khz)
{
    int dev = 0;
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipGetDeviceProperties(&prop, dev));
    if (compute_units) *compute_units = prop.multiProcessorCount;
    if (clock_khz) *clock_khz = prop.clockRate;
    return AGG_OK;
}

}  // extern "C"

/*
 * agg — AllGather-GEMM consumer and GEMM-ReduceScatter reducer for MI355X (gfx950).
 *
 * C ABI of libagg.so.  Plain pointers and sizes only.  Unless a parameter says
 * "host", every data pointer is a DEVICE pointer owned by the caller; the library
 * owns only what symm_alloc creates (the symmetric staging buffer, the signal
 * words and a few bookkeeping words).  Streams are hipStream_t passed as void*
 * (NULL = the default stream).  All work is enqueued asynchronously on the
 * caller's streams; only symm_alloc, symm_free and agg_status synchronise.
 * Nothing here falls back to the CPU.
 *
 * Every function returns AGG_OK (0) or a negative AGG_ERR_* code and has no other
 * effect when it fails; agg_strerror names a code.  Functions are not thread-safe
 * on one context; different contexts are independent.  A context carries one set of
 * arrival counters, slice counters and tile tables: two producers, two gemm_rs /
 * gemm_rs_scatter or two ag_moe_gemm launches of ONE context must not be in flight at the same time (order
 * them on a stream or with events, or use a context each); GEMMs with an AGG_B_KN operand share one buffer of
 * the context and are ordered by the library itself.
 *
 * Vocabulary (the paper's, Section 2.1 and Algorithms 1-3): W = WORLD_SIZE,
 * rank = RANK, T = symmetric buffer, S = signal array, L = a rank's local shard.
 */
#ifndef AGG_H
#define AGG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct agg_ctx agg_ctx;

enum {
    AGG_OK = 0,
    AGG_ERR_INVALID_ARG = -1,       /* null pointer, negative size, rank outside [0, W) ... */
    AGG_ERR_UNSUPPORTED_SHAPE = -2, /* K not a multiple of 64, M not a multiple of W, shard larger than T ... */
    AGG_ERR_MISALIGNED = -3,        /* a pointer or leading dimension breaks the 16-byte rule */
    AGG_ERR_HIP = -4,               /* a HIP runtime call failed (the HIP error is cleared) */
    AGG_ERR_TIMEOUT = -5,           /* a kernel gave up waiting for a signal (reported by agg_status) */
    AGG_ERR_NOMEM = -6,
    AGG_ERR_NOT_FOUND = -7,         /* the table of tuned configurations has no entry for the problem */
    AGG_ERR_IO = -8,                /* a file could not be opened, read or written */
    AGG_ERR_NOT_RESERVED = -9       /* a workspace the call needs has not been reserved, or is too small */
};

enum { AGG_BF16 = 0, AGG_F32 = 1 };          /* element type of an output matrix */
enum { AGG_B_NK = 0,                         /* B stored [N][K], K contiguous (weight layout of a linear layer): read in place */
       AGG_B_KN = 1 };                       /* B stored [K][N], N contiguous: transposed into a buffer of the context
                                                on the GEMM's stream before every GEMM (one more pass over B; the
                                                buffer is sized by agg_reserve_b_kn beforehand; calls with this
                                                layout on one context share it: a call on another stream than the
                                                previous one is made to wait, on the device, for that one's GEMM);
                                                ldb >= N */
enum { AGG_PRODUCER_KERNEL = 0,              /* copy kernel on a few CUs, release-stores the signals */
       AGG_PRODUCER_SDMA = 1,               /* copy engine (no compute units) + one 4-byte copy per signal */
       AGG_PRODUCER_LINKS = 2,              /* full mesh: every peer's shard on a "link" of its own, all at once, chunk by chunk */
       AGG_PRODUCER_SKIP_LOCAL = 0x100,     /* OR into mode: do not (re)copy the local shard in this call */
       AGG_PRODUCER_LOCAL_LAST = 0x200,     /* OR into mode: copy the local shard after the peers' instead of first */
       AGG_PRODUCER_NARROW = 0x400 };       /* OR into mode (copy kernel): workgroups of one wave instead of four, so that
                                               the copy takes a quarter of the register file and issue slots of the compute
                                               units it shares with the consumer (Section 3.8: few resources for communication);
                                               when the local shard is not copied first, the first shard to arrive is still
                                               copied by four-wave workgroups: the consumer's first round of tiles waits for it */

/* One signal word per AGG_SIGNAL_STRIDE int32 (each signal owns a 128-byte line). */
#define AGG_SIGNAL_STRIDE 32

/* ------------------------------------------------------------------------------------------------
 * Symmetric memory and signals (Section 2.1: symmetric memory, signal exchange).
 *
 * symm_alloc creates this rank's symmetric buffer T of world_size * shard_bytes bytes (shard r lives at
 * byte offset r * shard_bytes, the layout of Algorithms 1 and 2) and n_signals signal words, all zero.
 * A context carries an epoch, starting at 1: a signal counts as set when its value >= epoch, so
 * signal_reset only has to advance the epoch (no device work, nothing to race with) and a signal left
 * over from an earlier run can never satisfy a wait.  shard_bytes must be a multiple of 16.
 * n_signals >= world_size; signals are grouped per shard: chunk c of shard r is signal
 * r * (n_signals / world_size) + c, so n_signals must be a multiple of world_size.
 * symm_alloc and symm_free synchronise the device.
 */
int symm_alloc(agg_ctx** ctx, int world_size, int rank, size_t shard_bytes, int n_signals);
int symm_free(agg_ctx* ctx);
void* symm_staging(agg_ctx* ctx);            /* device pointer to T, borrowed */
int32_t* symm_signals(agg_ctx* ctx);         /* device pointer to S (signal i at S[i * AGG_SIGNAL_STRIDE]), borrowed */
int symm_epoch(agg_ctx* ctx);                /* current epoch (host value) */

/*
 * Two streams the context owns, for the communication part and the computation part (Section 2.3: the host puts
 * communication and computation on separate streams).  Kernels of streams that
 * share a hardware queue run one after the other, and a consumer launched ahead of its producer on such a pair
 * would wait for signals that cannot come (its waits are bounded, so it would time out, not hang).  Which queue
 * a stream gets cannot be chosen, so symm_alloc tries it out: it keeps the first of up to eight new streams on
 * which a one-thread kernel gets through while a one-thread kernel on the consumer stream is still waiting for it
 * (at most 0.5 ms per try).  Callers may use streams of their own instead; then they should launch the producer first.
 */
int symm_streams(agg_ctx* ctx, void** producer_stream, void** consumer_stream);

/*
 * Every signal is reset before every run of an overlapped function (Section 3.8, the autotuner's rule).
 * Advances the epoch; calls issued afterwards wait for, and set, the new epoch.  The caller orders the
 * previous run's kernels before the next run's producer (they share T).  `stream` is used only with
 * agg_set_device_epoch(ctx, 1).
 */
int signal_reset(agg_ctx* ctx, void* stream);

/*
 * Where the epoch lives.  0 (default): on the host; every launch takes the epoch as an argument when it is enqueued,
 * and signal_reset is host work only.  1: in a device word; signal_reset enqueues a one-thread kernel on `stream`
 * that advances it, and every kernel of this library (producers, signal_set, the GEMMs, the reducer) reads the epoch
 * from that word when it STARTS.  The caller then orders signal_reset before the launches of the run on their streams
 * (an event from the reset's stream to the producer's and the consumer's), and a whole run -- reset, arrival, gated
 * GEMM, join -- can be recorded into a HIP graph by stream capture and replayed: every replay is a run with a fresh
 * epoch.  (With the epoch on the host a replay would compare the signals with the epoch of the recording, which the
 * first run has already reached.)  Nothing this library enqueues for a run is a memset or an allocation (workspaces
 * are sized beforehand by the agg_reserve_* calls); the first launch of a tile configuration sets a function
 * attribute, so run once before recording.  In this mode gemm_rs and moe_rs order their reducer behind the whole GEMM with an event (a stream
 * wait on memory compares with a value fixed at enqueue time).  symm_epoch keeps counting the host's resets and does
 * not see replays.  Synchronises the device.
 */
int agg_set_device_epoch(agg_ctx* ctx, int on);

/* Set signal `index` to the current epoch on `stream` (a 4-byte release store by a one-thread kernel). */
int signal_set(agg_ctx* ctx, int index, void* stream);

/*
 * Bound every in-kernel wait: after `microseconds` without its signal a workgroup records a time-out,
 * every workgroup of that launch stops waiting, and the launch drains (its output is then undefined).
 * Default 2,000,000 (2 s).  0 is rejected: an unbounded wait can hang the GPU.
 */
int agg_set_wait_limit_us(agg_ctx* ctx, uint64_t microseconds);

/* Synchronises the device, then returns AGG_OK, or AGG_ERR_TIMEOUT if any launch on this context
 * since the last agg_status call gave up a wait (the record is cleared). */
int agg_status(agg_ctx* ctx);

/* ------------------------------------------------------------------------------------------------
 * Emulated AllGather arrival (Algorithm 2, pull mode, seen from this rank; on one GPU the "remote"
 * shards are other device buffers).
 *
 * remote_shards: HOST array of W device pointers; remote_shards[r] is rank r's local buffer L_r
 * (shard_bytes each).  First L_rank is copied to T + rank*shard_bytes and its signals are set (unless mode
 * carries AGG_PRODUCER_SKIP_LOCAL, for callers that deliver the shards over several calls); then, for
 * each r in arrival_order (HOST array of n_arrivals ranks, each != rank, no repeats; NULL = the rotated
 * order rank+1, rank+2, ... and n_arrivals is ignored), L_r is copied to T + r*shard_bytes chunk by chunk
 * and each chunk's signal is set (release) once the chunk has landed.  Shards not listed never arrive.
 * mode: AGG_PRODUCER_KERNEL uses `n_workgroups` workgroups (0 = one per compute unit) whose registers fit beside
 * the consumer's on every CU; AGG_PRODUCER_SDMA uses hipMemcpyAsync without compute units; AGG_PRODUCER_LINKS
 * (Section 3.7, full mesh) copies the local shard first and then all listed peers side by side, each on an equal
 * share of the workgroups, chunk after chunk, optionally held to agg_set_link_rate: chunk c of every peer then
 * arrives at about (c + 1) * chunk_bytes / rate, whatever the order of the list.
 */
int ag_producer_emulate(agg_ctx* ctx, const void* const* remote_shards, const int* arrival_order,
                        int n_arrivals, int mode, int n_workgroups, void* producer_stream);

/* ------------------------------------------------------------------------------------------------
 * AllGather-GEMM consumer (Section 2.3 / Figure 4: a tiled GEMM whose tiles wait on the signals of the
 * shards they read; Section 3.7: rank-rotated tile order, local shard first).
 *
 * C[M, N] = A[M, K] . B with A = T viewed as [M, K] bf16 row-major (lda = K; M = W * Ms, shard r = rows
 * [r*Ms, (r+1)*Ms), so shard_bytes must equal Ms*K*2), B bf16 in the layout b_layout names with leading
 * dimension ldb (elements), C row-major with leading dimension ldc (elements) of type c_dtype.
 * Accumulation is fp32; bf16 output is rounded to nearest even from the fp32 accumulator.
 * Each tile waits (acquire) for every signal covering its rows to reach the current epoch before its
 * first load of A.  Requirements: K % 64 == 0, M % W == 0; for AGG_B_NK ldb % 8 == 0 and B 16-byte aligned;
 * C aligned to its element size; M, N arbitrary (>= 0; 0 is a no-op).
 */
int ag_gemm(agg_ctx* ctx, int M, int N, int K,
            const void* B, int ldb, int b_layout,
            void* C, int ldc, int c_dtype, void* consumer_stream);

/* ------------------------------------------------------------------------------------------------
 * ReduceScatter reduction (Algorithm 3, stream 2): R = sum_{w=0}^{W-1} slot_w, fp32, in the order
 * w = 0, 1, .., W-1 starting from +0, whatever the arrival order.  Before reading slot w the kernel waits
 * for signal w * (n_signals / W) to reach the current epoch.
 * A waiting reducer occupies compute units: whatever raises the signals must be able to run beside it
 * (copies, signal_set and this library's producer can; a kernel that needs every register of a CU cannot).
 * slots: HOST array of W device pointers to fp32 [Ms, N] row-major (leading dimension N).
 * R: [Ms, N] of r_dtype, leading dimension ldr.  Ms * N must be a multiple of 4; slots 16-byte aligned.
 * n_workgroups: size of the (persistent) grid, 0 = the library's choice (three workgroups per two compute units).
 * With agg_set_rs_chunks(k > 1) the wait is per row chunk of a slot instead (see there).
 */
int rs_reduce(agg_ctx* ctx, int Ms, int N, const float* const* slots,
              void* R, int ldr, int r_dtype, int n_workgroups, void* stream);

/*
 * GEMM + ReduceScatter for one rank (Section 3.3, Algorithm 3; Section 4.1 "GEMM ReduceScatter").
 * Enqueues on gemm_stream the local partial product P[M, N] = A_local[M, Klocal] . B_local (bf16 in, fp32
 * out, un-gated), writing this rank's row slice [rank*Ms, (rank+1)*Ms) straight into slots[rank] (it is computed
 * last by default, first with agg_set_rs_own_slice_last(ctx, 0)); when that slice is complete its signal is set
 * (the producer signal of Algorithm 3).
 * The other rows go to P_other (fp32 [M, N], leading dimension N; rows of the own slice are not written;
 * may be NULL to skip computing them).  Enqueues on reduce_stream a stream-level wait for the own slot's
 * signal (it holds no compute unit, so the GEMM can always become resident) and then the reduction of
 * rs_reduce, which waits for every slot's signal and runs beside the rest of the GEMM.  Peers' slots "arrive" when the caller sets their signals
 * (signal_set, or a producer of the caller's own).
 */
int gemm_rs(agg_ctx* ctx, int M, int N, int Klocal,
            const void* A_local, int lda, const void* B_local, int ldb, int b_layout,
            const float* const* slots, float* P_other,
            void* R, int ldr, int r_dtype, void* gemm_stream, void* reduce_stream);

/*
 * Tuning (Section 3.8, the autotuner for overlapped kernels).  What is timed is the whole overlapped function:
 * signal_reset, ag_producer_emulate (rotated arrival order) on the context's producer stream, ag_gemm on its consumer
 * stream, join -- with the signals reset before every run, never a kernel repeated on its own.  Candidates: the four
 * tile shapes x both tile orders x three producer sizes (half, one and two workgroups per compute unit; one candidate
 * when the copy engines are used).  Each candidate runs once to warm up (the very first thirty times, so that the
 * chip's clocks have settled) and runs_per_config more times; the median run counts.  The best configuration is stored in the context (tile shape, tile order, producer
 * size used when ag_producer_emulate is called with n_workgroups = 0) and returned.  Synchronous.  On one GPU
 * there is no agreement between ranks to reach; on a node the ranks would exchange *out and take the slowest
 * rank's best.  C is overwritten.  Any error leaves the context's settings as they were.
 */
typedef struct agg_tune_result {
    int tile_config, tile_order, producer_workgroups, configs_tried;
    float best_ms;
} agg_tune_result;
int agg_autotune_ag_gemm(agg_ctx* ctx, int M, int N, int K, const void* B, int ldb, int b_layout,
                         void* C, int ldc, int c_dtype, const void* const* remote_shards, int producer_mode,
                         int runs_per_config, agg_tune_result* out);

/*
 * Table of tuned configurations (Section 3.8: tuning results are kept and reused).  Process-wide and thread-safe; the
 * key is (world size, M, N, K).  agg_autotune_ag_gemm enters every result it returns.  agg_tune_table_apply copies the
 * entry for (ctx's world size, M, N, K) into the context (tile shape, tile order, producer size), as the tuner itself
 * does at its end, or returns AGG_ERR_NOT_FOUND and leaves the context alone.  save writes the table as text (one
 * header line, then "W M N K tile_config tile_order producer_workgroups configs_tried best_ms" per entry; lines
 * starting with # are comments); load merges such a file into the table (entries of the file win) and returns the
 * number of entries read, AGG_ERR_IO if the file cannot be read, or AGG_ERR_INVALID_ARG for a file with a wrong
 * header, a malformed line or a value out of range -- the table is then left exactly as it was.  None of these calls
 * touches the GPU.
 */
int agg_tune_table_size(void);
int agg_tune_table_clear(void);
int agg_tune_table_put(int world_size, int M, int N, int K, const agg_tune_result* entry);
int agg_tune_table_get(int world_size, int M, int N, int K, agg_tune_result* out);
int agg_tune_table_save(const char* path);
int agg_tune_table_load(const char* path);
int agg_tune_table_apply(agg_ctx* ctx, int M, int N, int K);

/*
 * The GEMM half of GEMM + ReduceScatter with the scatter fused into its epilogue (Section 3.6, "Intra-node
 * ReduceScatter with Fusion"; Algorithm 3, stream 1): P[M, N] = A_local[M, Klocal] . B_local in fp32, cut into W row
 * slices of M / W rows.  Slice w is stored straight into slice_dst[w] (HOST array of W DEVICE pointers, each fp32
 * [M / W, N] row-major, 16-byte aligned -- on a node, rank w's slot for this rank) or, where slice_dst[w] is NULL,
 * into rows [w*Ms, (w+1)*Ms) of P_other (fp32 [M, N]; may be NULL when no entry of slice_dst is).  When the last tile
 * of slice w has been stored, *slice_signal[w] (HOST array of W DEVICE pointers to int32 signal words, or NULL, or
 * NULL entries) is set to this context's epoch with release semantics -- the notify that lets rank w's reducer read
 * its slot.  Slices are computed starting with first_slice, then first_slice + 1, ... (Section 3.7: a rank starts
 * with the slices that have to travel and keeps its own for last).  With several contexts on one GPU, one per
 * emulated rank, wired to each other's slots and signals, this runs Algorithm 3 end to end (launch the GEMMs before
 * the reducers then: the streams of many contexts share the device's few hardware queues, and a GEMM queued behind a
 * reducer that waits for its signal cannot start until that reducer's time limit).
 */
int gemm_rs_scatter(agg_ctx* ctx, int M, int N, int Klocal,
                    const void* A_local, int lda, const void* B_local, int ldb, int b_layout,
                    float* const* slice_dst, float* P_other, int32_t* const* slice_signal,
                    int first_slice, void* gemm_stream);

/* ------------------------------------------------------------------------------------------------
 * MoE AllGather grouped GEMM (Section 4.1 "AllGather MoE", Table 4; tensor parallel).
 * T holds the gathered tokens X[Ttok, K] (shard r = tokens [r*tpr, (r+1)*tpr)).  topk_ids: DEVICE int32
 * [Ttok, topk], distinct experts per token.  The (token, slot) pairs are ordered by (expert, token, slot);
 * Y[p, :] = X[token(p), :] . W_expert(p) for the p-th pair, Y [Ttok*topk, N] row-major of y_dtype.
 * weights: bf16 [E][N][K] (K contiguous per expert).  sorted_token / sorted_expert_offsets are DEVICE
 * outputs the call fills (int32 [Ttok*topk] and int32 [E+1]) and then uses; the caller may read them.
 * A tile lies inside one expert's segment and waits for the signals of the rows of T between its first and its
 * last token (tokens rise inside a segment, so that range holds every token of the tile).
 * Requirements: K % 64 == 0, Ttok % W == 0, shard_bytes == (Ttok / W) * K * 2, Ttok * K * 2 < 2 GiB, E <= 4096,
 * weights and topk_ids 16-byte aligned, ldy >= N.  Ids outside [0, E) are skipped: their pairs appear nowhere and
 * sorted_expert_offsets[E] is then smaller than Ttok * topk.  Rows of Y past sorted_expert_offsets[E] are not
 * written.  Routing and GEMM run on `stream`; routing does not depend on T and runs before any signal is awaited.
 * The call allocates nothing and does not synchronise: the tile table it builds lives in a workspace of the context
 * that agg_reserve_moe sizes beforehand (AGG_ERR_NOT_RESERVED otherwise).
 */
int ag_moe_gemm(agg_ctx* ctx, int Ttok, int topk, int E, int N, int K,
                const int32_t* topk_ids, const void* weights,
                int32_t* sorted_token, int32_t* sorted_expert_offsets,
                void* Y, int ldy, int y_dtype, void* stream);

/*
 * Workspaces of a context, sized ahead of the calls that use them; these two are the only calls besides symm_alloc that
 * allocate device memory (they synchronise the device; they only ever grow a workspace).  No GEMM, MoE or reducer call
 * allocates or synchronises: one that finds its workspace missing or too small returns AGG_ERR_NOT_RESERVED.
 *   agg_reserve_b_kn: the [N][K] copy of a B operand given as AGG_B_KN (ag_gemm, gemm_rs, gemm_rs_scatter).
 *   agg_reserve_moe : the routing's counters (66 KB, zeroed once) and the tile table of the grouped GEMM (ag_moe_gemm,
 *                     moe_rs) for problems of up to Ttok * topk pairs, E experts and N columns, whatever tile
 *                     configuration is chosen later.  The routing kernel's workgroups read one another's counts through
 *                     those counters and wait for them (bounded by the limit of agg_set_wait_limit_us, like every wait): a MoE
 *                     call is one launch of E workgroups of 1024 threads that all have to become resident in turn.
 */
int agg_reserve_b_kn(agg_ctx* ctx, int N, int K);
int agg_reserve_moe(agg_ctx* ctx, int Ttok, int topk, int E, int N);

/*
 * ag_moe_gemm for callers that cannot allocate device memory and cannot ask a context to (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, same result, but the routing's
 * counters and the tile table live in a fixed array of 1088 KiB in the library's own device image (one copy per GPU,
 * held until the process ends) instead of a reserved workspace.  The call allocates nothing, frees nothing and does
 * not synchronise.  It returns AGG_ERR_UNSUPPORTED_SHAPE when the table of the problem could exceed the array:
 * (Ttok * topk / 128 + E) * ceil(N / 128) entries of 32 bytes must fit in 32760 entries (the Table 4 shape needs
 * 3072).  All contexts on one GPU share the array, and it keeps the last call's contents (the counters return to their
 * rest state at the end of every call and every table entry a call reads it has written first, so nothing needs
 * clearing): two calls that overlap in time on one GPU race, whatever their contexts and streams -- order them.
 */
int ag_moe_gemm_static(agg_ctx* ctx, int Ttok, int topk, int E, int N, int K,
                       const int32_t* topk_ids, const void* weights,
                       int32_t* sorted_token, int32_t* sorted_expert_offsets,
                       void* Y, int ldy, int y_dtype, void* stream);

/*
 * Let ag_gemm read this rank's own shard from `local_shard` (DEVICE pointer to L_rank, [Ms][K] bf16, 16-byte aligned,
 * borrowed until reset with NULL) instead of from T: tiles that lie wholly inside the own shard then wait for nothing
 * and start before any copy has landed.  T is still completed by the producer; with AGG_PRODUCER_LOCAL_LAST the local
 * copy, which nobody waits for any more, is done after the peers'.  The caller must not modify L_rank while ag_gemm
 * runs.  Same result bit for bit.
 */
int agg_set_local_shard(agg_ctx* ctx, const void* local_shard);

/*
 * Order in which ag_gemm walks the m-tiles (Section 3.7).  AGG_ORDER_ROTATED (default): the local shard, then the
 * peers' shards whole, in pull order rank+1, rank+2, ... -- matches a producer that delivers one shard after the
 * other (a switched fabric).  AGG_ORDER_SUBCHUNK: the local shard, then the first chunk of every peer, the second
 * chunk of every peer, ... -- matches AGG_PRODUCER_LINKS (a full mesh, every peer on its own link).  It needs
 * shards and chunks that are whole numbers of tile rows and is otherwise ignored.  The result is the same bit for
 * bit in either order.
 */
enum { AGG_ORDER_ROTATED = 0, AGG_ORDER_SUBCHUNK = 1 };
int agg_set_tile_order(agg_ctx* ctx, int order);

/*
 * Granularity of the GEMM + ReduceScatter signals (Section 3.6: the scatter is asynchronous and the reduction starts
 * on what has arrived; Algorithm 3's notify / wait pair, taken per block of rows instead of per whole slice).  With
 * chunks = k > 1 every slice of M / W rows is cut into k row chunks of M / (W k) rows, each with a signal of its own:
 *   - gemm_rs_scatter raises slice_signal[w][c * AGG_SIGNAL_STRIDE] when chunk c of slice w is complete at its
 *     destination (so slice_signal[w] must point at k signal words spaced AGG_SIGNAL_STRIDE apart);
 *   - rs_reduce (and the reducers inside gemm_rs and moe_rs) waits for signal w * (n_signals / W) + c before its first
 *     read of chunk c of slot w, and reduces the first chunks while later ones are still being produced.  A workgroup
 *     waits for a chunk of ALL W slots before it adds that chunk up; the order of the additions is unchanged, so the
 *     result is the same bit for bit for every k.
 * Whoever plays the peers sets their k signals per slot.  1 <= k <= 16, k <= n_signals / W; M / W must be a multiple
 * of k and (M / (W k)) * N a multiple of 4 (else AGG_ERR_UNSUPPORTED_SHAPE from the launch).  Default 1.
 */
int agg_set_rs_chunks(agg_ctx* ctx, int chunks);

/*
 * Order of the slices inside gemm_rs (Section 3.7: a rank computes the slices that have to travel first and keeps its
 * own for last).  1 (default): the own slice last, as on a node; the reducer starts when the first chunk of the own
 * slice (agg_set_rs_chunks) is complete and reduces chunk by chunk behind the end of the GEMM.  0: the own slice
 * first, so that the reducer runs beside the whole rest of the GEMM (measured equally fast on one GPU, where the
 * peers' slots do not have to travel).  The results are the same bit for bit.
 */
int agg_set_rs_own_slice_last(agg_ctx* ctx, int on);

/* Pace of one link of AGG_PRODUCER_LINKS in GB/s (1e9 bytes per second); 0 (default) = as fast as the copy goes. */
int agg_set_link_rate(agg_ctx* ctx, double gigabytes_per_second);

/* ------------------------------------------------------------------------------------------------
 * MoE + ReduceScatter for one rank (Section 4.1 "MoE ReduceScatter", Table 5: grouped GEMM, top-k reduction, reduce
 * scatter; tensor parallel over K).
 * H: bf16 [Ttok*topk, Klocal], the routed rows in the order of ag_moe_gemm's output (pairs sorted by (expert, token,
 * slot)); weights2: bf16 [E][N][Klocal]; topk_ids as in ag_moe_gemm; gate: fp32 [Ttok, topk].
 *   Y[p, :] = H[p, :] . W2_expert(p)                       (Y: caller's fp32 workspace [Ttok*topk, N], overwritten; if
 *                                                           Z_other is NULL only the rows of this rank's tokens are
 *                                                           computed and stored, the other rows of Y keep what they held)
 *   Z[t, :] = sum_s gate[t, s] * Y[pair_pos[t*topk+s], :]  (fp32, slots in order; this rank's tokens go straight into
 *                                                           slots[rank], the others into row t of Z_other, or nowhere
 *                                                           if Z_other is NULL)
 *   R       = sum over w of slots[w]                        (rs_reduce: waits for every slot's signal; this call raises
 *                                                           the own slot's; the peers' arrive as for gemm_rs)
 * sorted_token [Ttok*topk], sorted_expert_offsets [E+1], pair_pos [Ttok*topk]: DEVICE int32 outputs the call fills and
 * uses (pair_pos[t*topk+s] = row of pair (t, s) in the sorted order).  Requirements: Klocal % 64 == 0, N % 4 == 0,
 * Ttok % W == 0, 16-byte aligned H, weights2, topk_ids, gate, Y, slots, Z_other.  GEMM, top-k reduction and the own
 * signal run on gemm_stream, the reducer on reduce_stream behind a stream-level wait for that signal.
 */
int moe_rs(agg_ctx* ctx, int Ttok, int topk, int E, int N, int Klocal,
           const void* H, const void* weights2, const int32_t* topk_ids, const float* gate,
           float* Y, int32_t* sorted_token, int32_t* sorted_expert_offsets, int32_t* pair_pos,
           const float* const* slots, float* Z_other, void* R, int ldr, int r_dtype,
           void* gemm_stream, void* reduce_stream);

/* Tile configuration of the GEMM kernels: -1 = chosen from the problem shape (default); bits 0-1 = tile shape
 * (0 = 256x224, 1 = 128x128, 2 = 256x256, 3 = 128x256), bit 2 = MFMA form of the main loop (0: 32x32x16, 4: 16x16x32,
 * what the automatic choice takes).  A tuning knob (Section 3.8).  All shapes of one MFMA form give the same bits
 * (the sum over K runs in the same order in all of them); the two forms group the sum over K differently (16 or 32
 * terms per instruction) and may differ in the last bits, both within the tolerance. */
int agg_set_tile_config(agg_ctx* ctx, int tile_config);

/*
 * Measured ceiling for the MFMA roofline: enqueues on `stream` a kernel in which every wave of one workgroup per
 * compute unit issues `iterations` x 56 v_mfma_f32_16x16x32_bf16 from registers (the GEMM's accumulator pattern, no
 * memory traffic); *flop receives the floating-point operations of the launch (host value, written at once).  The
 * caller times it.  constant_operands = 0: pseudo-random operands in the ranges of the benchmark's inputs (what real
 * data costs in power, hence in clock); 1: every operand element the same (the chip's best case).
 */
int agg_mfma_ceiling(agg_ctx* ctx, int iterations, int constant_operands, double* flop, void* stream);

const char* agg_strerror(int code);

/* Device facts the bench reports against (compute units, peak clock in kHz). */
int agg_device_info(int* compute_units, int* clock_khz);

#ifdef __cplusplus
}
#endif
#endif /* AGG_H */

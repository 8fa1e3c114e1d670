// Emulated AllGather arrival (Algorithm 2, pull mode): a copy kernel that moves the "remote" shards
// into the symmetric buffer chunk by chunk and release-stores each chunk's signal once every
// workgroup has finished its part of the chunk.  The kernel is written to need no LDS and few
// registers, so its waves fit beside the consumer's on any CU (Section 3.8, resource partition).
#include "agg_internal.h"

// Cache policy bits of the buffer instructions below, in the gfx940 / gfx950 encoding of the `aux` operand:
// 2 = nt (streaming) on the loads, 16 = sc1 (agent scope: written through this XCD's L2) on the stores.  The
// publication of a chunk rests on three properties of this hardware, not on the language's memory model:
//   1. a store with sc1 has reached memory (not just the writer's L2) when s_waitcnt vmcnt(0) returns;
//   2. the signal is a relaxed agent-scope store to a line of its own, issued after that wait, so it cannot overtake the data;
//   3. the consumer's acquire (buffer_inv sc1, executed by the wave that saw the signal) drops its XCD's L2 and its
//      CU's L1 copies of lines written elsewhere, so its loads of the chunk go to memory.
// Another target would need these re-checked: the build refuses it.
#if defined(__HIP_DEVICE_COMPILE__) && !defined(__gfx950__)
#error "the cache policy bits and the publication scheme of this file are those of gfx950"
#endif
#define AGG_PROD_LOAD_AUX 2

namespace agg {

typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;

// The grid is cut into teams of `team` workgroups.  Chunks are numbered in arrival order (all chunks of
// the first shard to arrive, then the next shard's, ...); team t copies chunks t, t + n_teams, ... and
// inside a team each workgroup copies one contiguous slice of the chunk; several chunks are in flight at
// once, which is also how a full mesh of links delivers (Section 3.7).
//
// The stores are write-through at agent scope (sc1): the data goes to memory instead of staying
// dirty in the L2 of the XCD the workgroup happens to run on, so no L2 write-back is needed before the
// signal -- a wait for the stores to complete is the release.  (An agent-scope release fence would write
// back the whole L2, once per workgroup and chunk, and that cost more than the copy itself.)  The consumer's
// acquire invalidates its own L2 lines, so its loads fetch the data from memory.
__global__ __launch_bounds__(256) void producer_kernel(const ProducerArgs a)
{
    const int tid = threadIdx.x;
    const unsigned span = blockDim.x * 16u;         // bytes one load instruction of the workgroup covers
    const int epoch = a.epoch_ptr ? __hip_atomic_load(a.epoch_ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : a.epoch;
    const int team = a.team;
    const int n_teams = gridDim.x / team;
    const int t = blockIdx.x / team, j = blockIdx.x - t * team;
    if (t >= n_teams) return;                       // left-over workgroups of a grid that is not a multiple of team
    const long long vec_per_chunk = a.chunk_bytes / 16;
    const long long per_wg = (vec_per_chunk + team - 1) / team;
    const long long lo = j * per_wg, hi = lo + per_wg < vec_per_chunk ? lo + per_wg : vec_per_chunk;
    const int n_chunks = a.n_jobs * a.chunks_per_shard;
    // cache policy bits: loads nt (streaming); stores sc1 = agent scope, written through this XCD's L2 so that the
    // consumer's XCDs find the data in memory (system scope or streaming stores were measured slightly slower
    // beside the GEMM)
    constexpr int NT = AGG_PROD_LOAD_AUX, WT = 16;
    for (int ch = t; ch < n_chunks; ch += n_teams) {
        const int job = ch / a.chunks_per_shard, c = ch - job * a.chunks_per_shard;
        const int r = a.rank_of[job];
        // this workgroup's slice [lo, hi) of the chunk, as buffers of at most (hi - lo) * 16 < 2^31 bytes
        const char* s = (const char*)a.src[job] + (c * vec_per_chunk + lo) * 16;
        char* d = a.T + (long long)r * a.shard_bytes + (c * vec_per_chunk + lo) * 16;
        const unsigned bytes = hi > lo ? (unsigned)((hi - lo) * 16) : 0u;
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(s), 0, bytes, 0x00020000);
        const __amdgpu_buffer_rsrc_t rd = __builtin_amdgcn_make_buffer_rsrc(d, 0, bytes, 0x00020000);
        // four independent 16-byte loads in flight per lane; out-of-range lanes of the last round load zero
        // and store nothing (the descriptors bound both)
        for (unsigned off = tid * 16u; off < bytes; off += 4u * span) {
            u32x4 v0 = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, NT);
            u32x4 v1 = __builtin_amdgcn_raw_buffer_load_b128(rs, off + span, 0, NT);
            u32x4 v2 = __builtin_amdgcn_raw_buffer_load_b128(rs, off + 2u * span, 0, NT);
            u32x4 v3 = __builtin_amdgcn_raw_buffer_load_b128(rs, off + 3u * span, 0, NT);
            __builtin_amdgcn_raw_buffer_store_b128(v0, rd, off, 0, WT);
            __builtin_amdgcn_raw_buffer_store_b128(v1, rd, off + span, 0, WT);
            __builtin_amdgcn_raw_buffer_store_b128(v2, rd, off + 2u * span, 0, WT);
            __builtin_amdgcn_raw_buffer_store_b128(v3, rd, off + 3u * span, 0, WT);
        }
        // signal: the last workgroup of the team to finish the chunk sets it (set_signal after the copy, Algorithm 2)
        __builtin_amdgcn_s_waitcnt(0);              // every store of this lane has completed
        __syncthreads();                            // ... of this workgroup
        if (tid == 0) {
            const int f = r * a.chunks_per_shard + c;
            const int prev = __hip_atomic_fetch_add(a.counters + f, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (prev == team - 1) {
                __hip_atomic_store(a.counters + f, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(a.flags + (long long)f * kSignalStride, epoch, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

// Full-mesh arrival (Section 3.7, the AMD case: a rank pulls from all its peers at once, one link each, and a
// shard arrives sub-chunk by sub-chunk).  Every job is one link served by link_wgs workgroups of its own; a link
// moves its shard chunk after chunk and sets each chunk's signal.  With ticks_per_byte > 0 a link is held to that
// rate: before each 16 KiB step a workgroup waits until the link's clock allows the bytes moved so far, so chunk c
// of every peer lands at about (c + 1) * chunk_bytes / rate after the start -- the arrival pattern of real links.
// The wait ends at a time computed beforehand, so it is bounded.
__global__ __launch_bounds__(256) void producer_links_kernel(const ProducerArgs a)
{
    const int tid = threadIdx.x;
    const unsigned span = 4096u;                    // bytes one load instruction of the workgroup covers (256 threads)
    const int epoch = a.epoch_ptr ? __hip_atomic_load(a.epoch_ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : a.epoch;
    const int link = blockIdx.x % a.n_jobs, j = blockIdx.x / a.n_jobs;
    if (j >= a.link_wgs) return;
    const long long t0 = wall_clock64();
    const long long vec_per_chunk = a.chunk_bytes / 16;
    const long long per_wg = (vec_per_chunk + a.link_wgs - 1) / a.link_wgs;
    const long long lo = j * per_wg, hi = lo + per_wg < vec_per_chunk ? lo + per_wg : vec_per_chunk;
    const unsigned bytes = hi > lo ? (unsigned)((hi - lo) * 16) : 0u;
    const int r = a.rank_of[link];
    constexpr int NT = AGG_PROD_LOAD_AUX, WT = 16;
    for (int c = 0; c < a.chunks_per_shard; ++c) {
        const char* s = (const char*)a.src[link] + (c * vec_per_chunk + lo) * 16;
        char* d = a.T + (long long)r * a.shard_bytes + (c * vec_per_chunk + lo) * 16;
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(s), 0, bytes, 0x00020000);
        const __amdgpu_buffer_rsrc_t rd = __builtin_amdgcn_make_buffer_rsrc(d, 0, bytes, 0x00020000);
        int step = 0;
        for (unsigned off = tid * 16u; off - tid * 16u < bytes; off += 4u * span, ++step) {
            if (a.ticks_per_byte > 0.0) {
                // bytes the link has moved when all its workgroups have done `step` steps of this chunk
                const double before = (double)c * (double)a.chunk_bytes + (double)step * 16384.0 * a.link_wgs;
                const long long target = t0 + (long long)(before * a.ticks_per_byte);
                while (wall_clock64() < target) __builtin_amdgcn_s_sleep(4);
            }
            u32x4 v0 = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, NT);
            u32x4 v1 = __builtin_amdgcn_raw_buffer_load_b128(rs, off + span, 0, NT);
            u32x4 v2 = __builtin_amdgcn_raw_buffer_load_b128(rs, off + 2u * span, 0, NT);
            u32x4 v3 = __builtin_amdgcn_raw_buffer_load_b128(rs, off + 3u * span, 0, NT);
            __builtin_amdgcn_raw_buffer_store_b128(v0, rd, off, 0, WT);
            __builtin_amdgcn_raw_buffer_store_b128(v1, rd, off + span, 0, WT);
            __builtin_amdgcn_raw_buffer_store_b128(v2, rd, off + 2u * span, 0, WT);
            __builtin_amdgcn_raw_buffer_store_b128(v3, rd, off + 3u * span, 0, WT);
        }
        if (a.ticks_per_byte > 0.0) {      // the chunk is not announced before the link could have delivered it
            const long long target = t0 + (long long)((double)(c + 1) * (double)a.chunk_bytes * a.ticks_per_byte);
            while (wall_clock64() < target) __builtin_amdgcn_s_sleep(4);
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (tid == 0) {
            const int f = r * a.chunks_per_shard + c;
            const int prev = __hip_atomic_fetch_add(a.counters + f, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (prev == a.link_wgs - 1) {
                __hip_atomic_store(a.counters + f, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(a.flags + (long long)f * kSignalStride, epoch, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

// value_ptr not null: the value is read from that device word (the context's epoch word) when the kernel runs
__global__ void signal_set_kernel(int* flag, int value, const int* value_ptr)
{
    if (value_ptr) value = __hip_atomic_load(value_ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(flag, value, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

// signal_reset with the epoch kept on the device: one thread, ordered by its stream like any other kernel
__global__ void epoch_advance_kernel(int* epoch_word)
{
    const int e = __hip_atomic_load(epoch_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(epoch_word, e + 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

// threads: 256 (four waves per workgroup) or 64 (one wave: a narrow producer that leaves the consumer more of every
// compute unit it shares)
hipError_t launch_producer(const ProducerArgs& a_in, int n_workgroups, int threads, hipStream_t stream)
{
    ProducerArgs a = a_in;
    // team size: slices of at least 64 KiB, at most the whole grid on one chunk
    long long team = a.chunk_bytes / 65536;
    if (team < 1) team = 1;
    if (team > n_workgroups) team = n_workgroups;
    a.team = (int)team;
    hipLaunchKernelGGL(producer_kernel, dim3(n_workgroups), dim3(threads), 0, stream, a);
    return hipGetLastError();
}

// All jobs of `a` are links that run side by side; the grid is shared out evenly among them.
hipError_t launch_producer_links(const ProducerArgs& a_in, int n_workgroups, hipStream_t stream)
{
    ProducerArgs a = a_in;
    if (a.n_jobs < 1) return hipSuccess;
    int per_link = n_workgroups / a.n_jobs;
    if (per_link < 1) per_link = 1;
    // no more workgroups on a link than it has 16 KiB steps in a chunk
    const long long steps = (a.chunk_bytes + 16383) / 16384;
    if (per_link > steps) per_link = (int)steps;
    a.link_wgs = per_link;
    hipLaunchKernelGGL(producer_links_kernel, dim3(per_link * a.n_jobs), dim3(256), 0, stream, a);
    return hipGetLastError();
}

// One thread waits (for at most `ticks` of the wall clock) until *flag >= value and writes what it saw to *seen:
// 1 = the value arrived, 2 = the wait ran out.  Used to find out whether two streams really run side by side.
__global__ void signal_probe_kernel(const int* flag, int value, long long ticks, int* seen)
{
    const long long t0 = wall_clock64();
    int ok = 0;
    while (!(ok = __hip_atomic_load(flag, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) >= value)) {
        if (wall_clock64() - t0 > ticks) break;
        __builtin_amdgcn_s_sleep(8);
    }
    __hip_atomic_store(seen, ok ? 1 : 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

hipError_t launch_signal_probe(const int* flag, int value, long long ticks, int* seen, hipStream_t stream)
{
    hipLaunchKernelGGL(signal_probe_kernel, dim3(1), dim3(1), 0, stream, flag, value, ticks, seen);
    return hipGetLastError();
}

hipError_t launch_signal_set(int* flag, int value, const int* value_ptr, hipStream_t stream)
{
    hipLaunchKernelGGL(signal_set_kernel, dim3(1), dim3(1), 0, stream, flag, value, value_ptr);
    return hipGetLastError();
}

hipError_t launch_epoch_advance(int* epoch_word, hipStream_t stream)
{
    hipLaunchKernelGGL(epoch_advance_kernel, dim3(1), dim3(1), 0, stream, epoch_word);
    return hipGetLastError();
}

}  // namespace agg

// Emulated AllGather arrival (Algorithm 2, pull mode): a copy kernel that moves the "remote" shards
// into the symmetric buffer chunk by chunk and release-stores each chunk's signal once every
// workgroup has finished its part of the chunk.  The kernel is written to need no LDS and few
// registers, so its waves fit beside the consumer's on any CU (Section 3.8, resource partition).
#include "agg_internal.h"

namespace agg {

typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;

__global__ __launch_bounds__(256) void producer_kernel(const ProducerArgs a)
{
    const int tid = threadIdx.x;
    const int nwg = gridDim.x;
    const long long vec_per_chunk = a.chunk_bytes / 16;
    const long long stride = (long long)nwg * 256;
    for (int j = 0; j < a.n_jobs; ++j) {
        const int r = a.rank_of[j];
        const u32x4* src = (const u32x4*)a.src[j];
        u32x4* dst = (u32x4*)(a.T + (long long)r * a.shard_bytes);
        for (int c = 0; c < a.chunks_per_shard; ++c) {
            const u32x4* s = src + c * vec_per_chunk;
            u32x4* d = dst + c * vec_per_chunk;
            long long i = (long long)blockIdx.x * 256 + tid;
            // four independent 16-byte loads in flight per lane; streaming (non-temporal) accesses keep
            // the copy from evicting the consumer's tiles from L2
            for (; i + 3 * stride < vec_per_chunk; i += 4 * stride) {
                u32x4 v0 = __builtin_nontemporal_load(s + i);
                u32x4 v1 = __builtin_nontemporal_load(s + i + stride);
                u32x4 v2 = __builtin_nontemporal_load(s + i + 2 * stride);
                u32x4 v3 = __builtin_nontemporal_load(s + i + 3 * stride);
                __builtin_nontemporal_store(v0, d + i);
                __builtin_nontemporal_store(v1, d + i + stride);
                __builtin_nontemporal_store(v2, d + i + 2 * stride);
                __builtin_nontemporal_store(v3, d + i + 3 * stride);
            }
            for (; i < vec_per_chunk; i += stride) __builtin_nontemporal_store(__builtin_nontemporal_load(s + i), d + i);
            // signal: the last workgroup to finish the chunk sets it (set_signal after the copy, Algorithm 2)
            __syncthreads();
            if (tid == 0) {
                const int f = r * a.chunks_per_shard + c;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
                const int prev = __hip_atomic_fetch_add(a.counters + f, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
                if (prev == nwg - 1) {
                    __hip_atomic_store(a.counters + f, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(a.flags + (long long)f * kSignalStride, a.epoch, __ATOMIC_RELEASE,
                                       __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
    }
}

__global__ void signal_set_kernel(int* flag, int value)
{
    __hip_atomic_store(flag, value, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

hipError_t launch_producer(const ProducerArgs& a, int n_workgroups, hipStream_t stream)
{
    hipLaunchKernelGGL(producer_kernel, dim3(n_workgroups), dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_signal_set(int* flag, int value, hipStream_t stream)
{
    hipLaunchKernelGGL(signal_set_kernel, dim3(1), dim3(1), 0, stream, flag, value);
    return hipGetLastError();
}

}  // namespace agg

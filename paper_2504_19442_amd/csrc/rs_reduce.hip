// ReduceScatter reduction (Algorithm 3, stream 2): R = sum over w = 0..W-1 of slot_w, fp32, added in
// that order starting from +0 whatever order the slots arrive in, so the result is bit-identical
// across arrival orders.  Each workgroup waits (acquire) for slot w's signal before its first read of
// slot w.  The kernel is bandwidth bound: W reads and one write per element, 16 bytes per lane per
// access; ordinary loads (streaming-hinted loads measured 10 % slower here), streaming stores.
#include "agg_internal.h"

namespace agg {

typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;


__device__ inline bool wait_signal(const int* fp, int epoch, long long ticks, int* err)
{
    const long long t0 = wall_clock64();
    while (__hip_atomic_load(fp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < epoch) {
        if (__hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0 || wall_clock64() - t0 > ticks) {
            __hip_atomic_store(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return false;
        }
        __builtin_amdgcn_s_sleep(1);
    }
    return true;
}

__device__ inline void store_out(const ReduceArgs& a, long long i, f32x4 v)
{
    long long off;
    if (a.row_vec4) {
        const long long row = i / a.row_vec4;
        off = row * a.ldr + (i - row * a.row_vec4) * 4;
    } else {
        off = i * 4;
    }
    if (a.r_is_f32) {
        __builtin_nontemporal_store(v, (f32x4*)((float*)a.R + off));
    } else {
        bf16x4 o;
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = (__bf16)v[k];
        *(bf16x4*)((__bf16*)a.R + off) = o;
    }
}

// WT > 0: the world size is the compile-time constant WT (loops over slots unroll, all loads of a block are in
// flight together); WT == 0: any world size.
template <int WT, int RU>   // RU = float4 per lane per slot and block
__global__ __launch_bounds__(256) void reduce_kernel(const ReduceArgs a)
{
    const int tid = threadIdx.x;
    const int W = WT > 0 ? WT : a.W;
    const int epoch = a.epoch_ptr ? __hip_atomic_load(a.epoch_ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : a.epoch;
    const long long stride = (long long)gridDim.x * 256;
    int seen = 0;                      // slots 0..seen-1 are known to have arrived (uniform over the workgroup)
    int chunks_seen = 0;               // chunked slots: row chunks 0..chunks_seen-1 of EVERY slot have arrived
    for (long long base = (long long)blockIdx.x * 256 + tid; base - tid < a.n_vec4; base += stride * RU) {
        f32x4 acc[RU];
#pragma unroll
        for (int u = 0; u < RU; ++u) acc[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (a.chunks > 1) {
            // Slots that arrive in row chunks, each chunk with a signal of its own: a workgroup walks the rows
            // upwards, so before it enters a chunk it waits for that chunk (and any it skipped) of all W slots,
            // and the reduction of the first chunks runs while the later ones are still being produced.
            long long last = (base - tid) + (long long)(RU - 1) * stride + 255;
            if (last >= a.n_vec4) last = a.n_vec4 - 1;
            const int need = (int)(last / a.chunk_vec4);
            if (need >= chunks_seen) {
                int ok = 1;
                if (tid == 0) {
                    for (int c = chunks_seen; ok && c <= need; ++c)
                        for (int w = 0; ok && w < W; ++w)
                            ok = wait_signal(a.flags + ((long long)w * a.flag_step + c) * kSignalStride, epoch,
                                             a.wait_ticks, a.err);
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
                }
                if (__syncthreads_or(!ok)) return;
                chunks_seen = need + 1;
            }
        }
        if (a.chunks <= 1 && seen < W) {
            // slots still to arrive: take them one by one in the order of Algorithm 3.  A wait that ends also
            // looks at the signals after it, so that one acquire (an L2 invalidate) covers all that are set.
            for (int w = 0; w < W; ++w) {
                if (w >= seen) {
                    int ok = 1, upto = w + 1;
                    if (tid == 0) {
                        ok = wait_signal(a.flags + (long long)w * a.flag_step * kSignalStride, epoch, a.wait_ticks, a.err);
                        while (ok && upto < W &&
                               __hip_atomic_load(a.flags + (long long)upto * a.flag_step * kSignalStride, __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT) >= epoch)
                            ++upto;
                        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
                    }
                    upto = __builtin_amdgcn_readfirstlane(upto);      // thread 0 is lane 0 of wave 0
                    __shared__ int s_upto;
                    if (tid == 0) s_upto = upto;
                    if (__syncthreads_or(!ok)) return;
                    seen = s_upto;
                    __syncthreads();
                }
                const f32x4* s = (const f32x4*)a.slot[w];
#pragma unroll
                for (int u = 0; u < RU; ++u) {
                    const long long i = base + u * stride;
                    const f32x4 v = (i < a.n_vec4) ? s[i] : f32x4{0.f, 0.f, 0.f, 0.f};
                    acc[u] = acc[u] + v;                              // R = R + T[w], one fp32 rounding each
                }
            }
        } else {
            // every slot has arrived: all loads of the block first, then the additions in slot order
            if constexpr (WT > 0) {
                f32x4 v[WT][RU];
#pragma unroll
                for (int w = 0; w < WT; ++w)
#pragma unroll
                    for (int u = 0; u < RU; ++u) {
                        const long long i = base + u * stride;
                        v[w][u] = (i < a.n_vec4) ? ((const f32x4*)a.slot[w])[i]
                                                 : f32x4{0.f, 0.f, 0.f, 0.f};
                    }
#pragma unroll
                for (int w = 0; w < WT; ++w)
#pragma unroll
                    for (int u = 0; u < RU; ++u) acc[u] = acc[u] + v[w][u];
            } else {
                for (int w = 0; w < W; ++w) {
                    const f32x4* s = (const f32x4*)a.slot[w];
#pragma unroll
                    for (int u = 0; u < RU; ++u) {
                        const long long i = base + u * stride;
                        const f32x4 v = (i < a.n_vec4) ? s[i] : f32x4{0.f, 0.f, 0.f, 0.f};
                        acc[u] = acc[u] + v;
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            const long long i = base + u * stride;
            if (i < a.n_vec4) store_out(a, i, acc[u]);
        }
    }
}

// beside_gemm: the launch is meant to run on the same compute units as the GEMM kernel, whose waves leave 64 vector
// registers per SIMD lane free: only kernels of at most 64 registers per lane fit there (a bigger one starts only where
// a GEMM workgroup has finished).  All variants but <8, 2> are that small.
hipError_t launch_reduce(const ReduceArgs& a, int n_workgroups, hipStream_t stream, bool beside_gemm)
{
    if (a.W == 8 && beside_gemm) {
        hipLaunchKernelGGL((reduce_kernel<8, 1>), dim3(n_workgroups), dim3(256), 0, stream, a);
        return hipGetLastError();
    }
    switch (a.W) {
        case 8: hipLaunchKernelGGL((reduce_kernel<8, 2>), dim3(n_workgroups), dim3(256), 0, stream, a); break;
        case 4: hipLaunchKernelGGL((reduce_kernel<4, 2>), dim3(n_workgroups), dim3(256), 0, stream, a); break;
        case 2: hipLaunchKernelGGL((reduce_kernel<2, 4>), dim3(n_workgroups), dim3(256), 0, stream, a); break;
        default: hipLaunchKernelGGL((reduce_kernel<0, 2>), dim3(n_workgroups), dim3(256), 0, stream, a); break;
    }
    return hipGetLastError();
}

}  // namespace agg

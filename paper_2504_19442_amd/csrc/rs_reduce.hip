// ReduceScatter reduction (Algorithm 3, stream 2): R = sum over w = 0..W-1 of slot_w, fp32, added in
// that order starting from +0 whatever order the slots arrive in, so the result is bit-identical
// across arrival orders.  Each workgroup waits (acquire) for slot w's signal before its first read of
// slot w.  The kernel is bandwidth bound: W reads and one write per element, 16 bytes per lane per
// access, streaming loads.
#include "agg_internal.h"

namespace agg {

typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;

constexpr int RU = 4;   // float4 per lane per slot kept in flight

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

__global__ __launch_bounds__(256) void reduce_kernel(const ReduceArgs a)
{
    const int tid = threadIdx.x;
    const long long stride = (long long)gridDim.x * 256;
    int seen = 0;                      // slots 0..seen-1 are known to have arrived
    for (long long base = (long long)blockIdx.x * 256 + tid; base - tid < a.n_vec4; base += stride * RU) {
        f32x4 acc[RU];
#pragma unroll
        for (int u = 0; u < RU; ++u) acc[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int w = 0; w < a.W; ++w) {
            if (w >= seen) {           // uniform over the workgroup: `seen` only changes here
                int ok = 1;
                if (tid == 0) ok = wait_signal(a.flags + (long long)w * a.flag_step * kSignalStride, a.epoch, a.wait_ticks, a.err);
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
                if (__syncthreads_or(!ok)) return;
                seen = w + 1;
            }
            const f32x4* s = (const f32x4*)a.slot[w];
            f32x4 v[RU];
#pragma unroll
            for (int u = 0; u < RU; ++u) {
                const long long i = base + u * stride;
                v[u] = (i < a.n_vec4) ? __builtin_nontemporal_load(s + i) : f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int u = 0; u < RU; ++u) acc[u] = acc[u] + v[u];      // R = R + T[w], one fp32 rounding each
        }
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            const long long i = base + u * stride;
            if (i < a.n_vec4) store_out(a, i, acc[u]);
        }
    }
}

hipError_t launch_reduce(const ReduceArgs& a, int n_workgroups, hipStream_t stream)
{
    hipLaunchKernelGGL(reduce_kernel, dim3(n_workgroups), dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace agg

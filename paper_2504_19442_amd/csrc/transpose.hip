// B given as [K][N] (N contiguous) -> the [N][K] (K contiguous) form the GEMM kernel loads whole 128-byte lines
// of.  64 x 64 tiles through LDS, reads and writes both along the contiguous dimension.
#include "agg_internal.h"

namespace agg {

__global__ __launch_bounds__(256) void transpose_kn_kernel(const uint16_t* __restrict__ B_kn, long long ldb, int K, int N,
                                                           uint16_t* __restrict__ B_nk)
{
    __shared__ uint16_t tile[64][66];
    const int k0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;           // 64 x 4
    for (int r = ty; r < 64; r += 4) {
        const int k = k0 + r, n = n0 + tx;
        tile[r][tx] = (k < K && n < N) ? B_kn[(long long)k * ldb + n] : (uint16_t)0;
    }
    __syncthreads();
    for (int r = ty; r < 64; r += 4) {
        const int n = n0 + r, k = k0 + tx;
        if (n < N && k < K) B_nk[(long long)n * K + k] = tile[tx][r];
    }
}

hipError_t launch_transpose_kn(const uint16_t* B_kn, long long ldb, int K, int N, uint16_t* B_nk, hipStream_t stream)
{
    hipLaunchKernelGGL(transpose_kn_kernel, dim3((N + 63) / 64, (K + 63) / 64), dim3(256), 0, stream, B_kn, ldb, K, N, B_nk);
    return hipGetLastError();
}

}  // namespace agg

// Reduction of split weight-gradient tiles, shared by the backward passes.
#pragma once
#include "common.h"
#include "gemm_mfma.h"

namespace uoe {

// partial [sets*n*splits][M][N] fp32 -> storage dtype, the parts added in order and rounded once.
// Set s goes to dst[s], stored as [n][M][N] or transposed as [n][N][M].  32x32 tiles through LDS.
struct WgradReduceArgs {
    const float *partial;
    uint16_t *dst[4];
    int transposed[4];
    int n, M, N, splits;
};

template <int UNUSED = 0> __global__ __launch_bounds__(256) void wgrad_reduce_kernel(WgradReduceArgs a)
{
    __shared__ float tile[32][33];
    const int set = blockIdx.z / a.n, e = blockIdx.z - set * a.n, r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const float *src = a.partial + (size_t)blockIdx.z * a.splits * a.M * a.N;
    for (int i = ty; i < 32; i += 8) {
        float v = 0.f;
        if (r0 + i < a.M && c0 + tx < a.N)
            for (int j = 0; j < a.splits; ++j) v += src[((size_t)j * a.M + r0 + i) * a.N + c0 + tx];
        tile[i][tx] = v;
    }
    __syncthreads();
    uint16_t *dst = a.dst[set];
    const bool tr = a.transposed[set] != 0;
    for (int i = ty; i < 32; i += 8) {
        if (tr) {
            if (c0 + i < a.N && r0 + tx < a.M)
                dst[((size_t)e * a.N + c0 + i) * a.M + r0 + tx] = (uint16_t)(pack2_bf16(tile[tx][i], 0.f) & 0xFFFFu);
        } else if (r0 + i < a.M && c0 + tx < a.N)
            dst[((size_t)e * a.M + r0 + i) * a.N + c0 + tx] = (uint16_t)(pack2_bf16(tile[i][tx], 0.f) & 0xFFFFu);
    }
}

static inline hipError_t launch_wgrad_reduce(const WgradReduceArgs &a, int sets, hipStream_t st)
{
    hipLaunchKernelGGL((wgrad_reduce_kernel<0>), dim3((a.N + 31) / 32, (a.M + 31) / 32, sets * a.n), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace uoe

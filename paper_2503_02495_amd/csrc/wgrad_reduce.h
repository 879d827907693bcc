// Reduction of split-K weight-gradient tiles, shared by the backward passes.
#pragma once
#include "common.h"
#include "gemm_mfma.h"

namespace uoe {

// partial [n*splits][M][N] fp32 -> storage dtype, the ranges added in order and rounded once.
// The M rows are PARTS consecutive blocks of M/PARTS rows, block p going to dst[p]; each block is
// stored as [n][M/PARTS][N], or transposed as [n][N][M/PARTS].  32x32 tiles through LDS.
struct WgradReduceArgs {
    const float *partial;
    uint16_t *dst[3];
    int M, N, splits, transposed, parts;
};

template <int UNUSED = 0> __global__ __launch_bounds__(256) void wgrad_reduce_kernel(WgradReduceArgs a)
{
    __shared__ float tile[32][33];
    const int e = blockIdx.z, r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int mp = a.M / a.parts;  // a multiple of 32: a tile never straddles two blocks
    for (int i = ty; i < 32; i += 8) {
        float v = 0.f;
        if (r0 + i < a.M && c0 + tx < a.N)
            for (int j = 0; j < a.splits; ++j) v += a.partial[(((size_t)e * a.splits + j) * a.M + r0 + i) * a.N + c0 + tx];
        tile[i][tx] = v;
    }
    __syncthreads();
    const int part = r0 / mp, rr0 = r0 - part * mp;
    uint16_t *dst = a.dst[part];
    for (int i = ty; i < 32; i += 8) {
        if (a.transposed) {
            if (c0 + i < a.N && r0 + tx < a.M)
                dst[((size_t)e * a.N + c0 + i) * mp + rr0 + tx] = (uint16_t)(pack2_bf16(tile[tx][i], 0.f) & 0xFFFFu);
        } else if (r0 + i < a.M && c0 + tx < a.N)
            dst[((size_t)e * mp + rr0 + i) * a.N + c0 + tx] = (uint16_t)(pack2_bf16(tile[i][tx], 0.f) & 0xFFFFu);
    }
}

static inline hipError_t launch_wgrad_reduce(const WgradReduceArgs &a, int n, hipStream_t st)
{
    hipLaunchKernelGGL((wgrad_reduce_kernel<0>), dim3((a.N + 31) / 32, (a.M + 31) / 32, n), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace uoe

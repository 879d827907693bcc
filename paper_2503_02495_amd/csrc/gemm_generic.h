// Vector-ALU grouped GEMM engine: fp32 FMA on LDS tiles, any storage type, any problem from
// problems.h.  This is the engine of the fp32 storage path and the fallback for shapes the MFMA
// engine does not tile; it favours generality over speed.
// Tile 64x64x8, 256 threads, 4x4 outputs per thread.  grid = (ceil(N/64), ceil(maxM/64), groups).
#pragma once
#include "common.h"

namespace uoe {

template <typename T, typename P>
__global__ __launch_bounds__(256) void gemm_generic_kernel(P p)
{
    constexpr int BM = 64, BN = 64, BK = 8;
    __shared__ float As[BK][BM + 4];
    __shared__ float Bs[BK][BN + 4];
    const int g = blockIdx.z;
    const int M = p.rows(g), N = p.ncols(), K = p.kdim(g);
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    if (m0 >= M) return;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;

    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    const int kseg = p.kseg();
    const long bstride = p.b_stride();
    for (int k0 = 0; k0 < K; k0 += BK) {
        const int seg = k0 / kseg, off = k0 - seg * kseg;
        if (tid < 64) {  // A: one row of 8 k per thread
            float v[8];
            const int r = m0 + tid;
            if (r < M) load8(p.a_seg_ptr(g, r, seg) + off, v);
            else
#pragma unroll
                for (int q = 0; q < 8; ++q) v[q] = 0.f;
#pragma unroll
            for (int q = 0; q < 8; ++q) As[q][tid] = v[q];
        } else if (tid < 128) {  // B: 8 k-rows x 8 column segments of 8
            const int idx = tid - 64, kk = idx >> 3, cseg = idx & 7;  // cseg: column chunk, not a K segment
            float v[8];
            const int nn = n0 + cseg * 8;
            if (nn < N) load8(p.b_seg_ptr(g, seg, nn) + (long)(off + kk) * bstride, v);
            else
#pragma unroll
                for (int q = 0; q < 8; ++q) v[q] = 0.f;
#pragma unroll
            for (int q = 0; q < 8; ++q) Bs[kk][cseg * 8 + q] = v[q];
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; ++kk) {
            float av[4], bv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) bv[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int nn = n0 + tx * 4 + j;
        if (nn >= N) continue;
        const auto cc = p.col_ctx(g, nn);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = m0 + ty * 4 + i;
            if (r < M) p.store(g, r, nn, acc[i][j], cc);
        }
    }
}

template <typename T, typename P>
static hipError_t launch_gemm_generic(const P &p, int groups, int max_rows, int ncols, hipStream_t st)
{
    if (groups <= 0 || max_rows <= 0 || ncols <= 0) return hipSuccess;
    dim3 grid((ncols + 63) / 64, (max_rows + 63) / 64, groups);
    hipLaunchKernelGGL((gemm_generic_kernel<T, P>), grid, dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace uoe

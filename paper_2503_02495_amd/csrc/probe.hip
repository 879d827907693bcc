// Measurement aids: what this GPU delivers for the three elementary access patterns the layer's
// kernels are made of, so that a kernel's achieved rate can be read against a measured ceiling as
// well as against the published peak, and so that hardware byte counters can be calibrated on a
// transfer of known size.  None of these is a step of the layer.
//   probe_copy : dst[i] = src[i], 16 bytes per lane, grid-stride (reads n bytes, writes n bytes)
//   probe_read : reads n bytes, 16 bytes per lane, grid-stride, and folds them into one word per
//                workgroup (so the loads cannot be dropped); writes almost nothing
//   probe_mfma : every wave keeps 8 independent v_mfma_f32_32x32x16_bf16 accumulators busy for
//                `iters` rounds on operand fragments it loaded once (no memory traffic in the loop)
#include "common.h"

namespace uoe {

__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * 256 * 4;
    for (size_t i = (size_t)blockIdx.x * 256 * 4 + threadIdx.x; i < n16; i += stride) {
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i + u * 256 < n16) v[u] = src[i + u * 256];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i + u * 256 < n16) dst[i + u * 256] = v[u];
    }
}

__global__ __launch_bounds__(256) void probe_read_kernel(const uint4 *__restrict__ src, size_t n16, uint32_t *sink)
{
    const size_t stride = (size_t)gridDim.x * 256 * 8;
    uint32_t acc = 0;
    for (size_t i = (size_t)blockIdx.x * 256 * 8 + threadIdx.x; i < n16; i += stride) {
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = i + u * 256 < n16 ? src[i + u * 256] : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc ^= __shfl_xor(acc, off, 64);
    __shared__ uint32_t part[4];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = part[0] ^ part[1] ^ part[2] ^ part[3];
}

typedef __bf16 pb_bf16x8 __attribute__((ext_vector_type(8)));
typedef float pb_f32x16 __attribute__((ext_vector_type(16)));

// operands: 6 fragments of 64 lanes x 16 bytes (4 for the first MFMA operand, 2 for the second)
__global__ __launch_bounds__(256) void probe_mfma_kernel(const uint4 *__restrict__ operands, int iters, float *sink)
{
    const int lane = threadIdx.x & 63;
    pb_bf16x8 a[4], b[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = __builtin_bit_cast(pb_bf16x8, operands[i * 64 + lane]);
#pragma unroll
    for (int i = 0; i < 2; ++i) b[i] = __builtin_bit_cast(pb_bf16x8, operands[(4 + i) * 64 + lane]);
    pb_f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) s += acc[i][j][q];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

hipError_t launch_probe_copy(const void *src, void *dst, size_t bytes, hipStream_t st)
{
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    const size_t want = (n16 + 1023) / 1024;
    const unsigned grid = (unsigned)(want < 256 * 32 ? want : 256 * 32);
    hipLaunchKernelGGL(probe_copy_kernel, dim3(grid), dim3(256), 0, st, static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), n16);
    return hipGetLastError();
}

hipError_t launch_probe_read(const void *src, size_t bytes, uint32_t *sink, hipStream_t st)
{
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    const size_t want = (n16 + 2047) / 2048;
    const unsigned grid = (unsigned)(want < PROBE_READ_BLOCKS ? want : PROBE_READ_BLOCKS);
    hipLaunchKernelGGL(probe_read_kernel, dim3(grid), dim3(256), 0, st, static_cast<const uint4 *>(src), n16, sink);
    return hipGetLastError();
}

hipError_t launch_probe_mfma(const void *operands, int iters, float *sink, hipStream_t st)
{
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(PROBE_MFMA_BLOCKS), dim3(256), 0, st, static_cast<const uint4 *>(operands), iters, sink);
    return hipGetLastError();
}

}  // namespace uoe

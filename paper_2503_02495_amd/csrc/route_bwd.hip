// Backward pass of the two routers (Eq. 21 and Eq. 13-14) for given gradients of their gates.
//   expert router: z = W_E vec(x), g = softmax_n(z):  dz = g * (dg - sum_i g_i dg_i),
//                  dW_E = dz^T vec(x),  d_x += dz W_E
//   data router:   L = (x W_B)^T W_A per sample, gate = softmax over experts for each patch:
//                  dL = gate * (dgate - sum_i gate_i dgate_i),  U = W_A dL^T [l,n],
//                  dW_A = sum_b (x W_B) dL,  dW_B = sum_b x^T U,  d_x += U W_B^T
// All of it is memory-bound streaming over x, W_E and d_x with n <= 32 outputs per element, so it
// runs on the vector ALU in fp32 (no contraction here is large enough for the matrix cores: K is
// b, n or m).  d_x is read, updated and written in place (it arrives holding the block's own
// gradient).  Summation orders are fixed: no atomics.
#include "common.h"

namespace uoe {

template <typename T> __device__ __forceinline__ void store8(T *p, const float (&v)[8]);
template <> __device__ __forceinline__ void store8<float>(float *p, const float (&v)[8])
{
    *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4 *>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
template <> __device__ __forceinline__ void store8<bf16_t>(bf16_t *p, const float (&v)[8])
{
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) w[e] = (uint32_t)f32_to_bf16_bits(v[2 * e]) | ((uint32_t)f32_to_bf16_bits(v[2 * e + 1]) << 16);
    *reinterpret_cast<uint4 *>(p) = make_uint4(w[0], w[1], w[2], w[3]);
}

// W_E and its gradient are read or written once per call and are larger than the memory-side cache on the
// big shapes: with ONCE (chosen per launch, stream_once) their 16-byte accesses carry the non-temporal hint,
// so that they do not push x and d_x out of the caches.  fp32 storage keeps the plain accesses.
template <bool ONCE> __device__ __forceinline__ void load8_w(const float *p, float (&o)[8]) { load8(p, o); }
template <bool ONCE> __device__ __forceinline__ void load8_w(const bf16_t *p, float (&o)[8])
{
    const uint4 a = load16<ONCE>(p);
    o[0] = __uint_as_float(a.x << 16); o[1] = __uint_as_float(a.x & 0xFFFF0000u);
    o[2] = __uint_as_float(a.y << 16); o[3] = __uint_as_float(a.y & 0xFFFF0000u);
    o[4] = __uint_as_float(a.z << 16); o[5] = __uint_as_float(a.z & 0xFFFF0000u);
    o[6] = __uint_as_float(a.w << 16); o[7] = __uint_as_float(a.w & 0xFFFF0000u);
}
template <bool ONCE> __device__ __forceinline__ void store8_w(float *p, const float (&v)[8]) { store8<float>(p, v); }
template <bool ONCE> __device__ __forceinline__ void store8_w(bf16_t *p, const float (&v)[8])
{
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) w[e] = (uint32_t)f32_to_bf16_bits(v[2 * e]) | ((uint32_t)f32_to_bf16_bits(v[2 * e + 1]) << 16);
    store16<ONCE>(p, make_uint4(w[0], w[1], w[2], w[3]));
}

// Softmax backward of both routers: block = sample.  dz_i = g_i (dg_i - sum_j g_j dg_j) is
// evaluated as g_i * sum_j g_j (dg_i - dg_j) (the gates sum to one): with one gate close to 1 the
// first form subtracts two nearly equal numbers, the second adds small terms of mixed sign only.
__global__ __launch_bounds__(64) void route_bwd_softmax_kernel(RouteBwdArgs a)
{
    const int bb = blockIdx.x, tid = threadIdx.x;
    if (a.w_e && blockIdx.y == 0 && tid < a.n) {
        const float *g = a.g_e + (size_t)bb * a.n, *dg = a.d_g_e + (size_t)bb * a.n;
        const float mine = dg[tid];
        float s = 0.f;
        for (int i = 0; i < a.n; ++i) s = fmaf(g[i], mine - dg[i], s);
        a.dz[(size_t)bb * a.n + tid] = g[tid] * s;
    }
    if (a.w_b)
        for (int j = blockIdx.y * 64 + tid; j < a.m; j += 64 * gridDim.y) {
            const float *g = a.g_p + (size_t)bb * a.n * a.m + j, *dg = a.d_g_p + (size_t)bb * a.n * a.m + j;
            for (int i = 0; i < a.n; ++i) {
                const float mine = dg[(size_t)i * a.m];
                float s = 0.f;
                for (int q = 0; q < a.n; ++q) s = fmaf(g[(size_t)q * a.m], mine - dg[(size_t)q * a.m], s);
                a.dl[((size_t)bb * a.n + i) * a.m + j] = g[(size_t)i * a.m] * s;
            }
        }
}

// dW_E[i, q] = sum_b dz[b,i] x[b,q]: thread = 8 consecutive q, block.y = a group of 8 experts
template <typename T, bool ONCE> __global__ __launch_bounds__(256) void route_bwd_wexpert_kernel(RouteBwdArgs a)
{
    constexpr int EG = 8;
    __shared__ float dzs[128 * EG];
    const long ld = (long)a.l * a.d, q = ((long)blockIdx.x * 256 + threadIdx.x) * 8;
    const int e0 = blockIdx.y * EG, ne = min(EG, a.n - e0);
    for (int idx = threadIdx.x; idx < a.b * EG; idx += 256) {
        const int bb = idx / EG, e = idx - bb * EG;
        dzs[idx] = e < ne ? a.dz[(size_t)bb * a.n + e0 + e] : 0.f;
    }
    __syncthreads();
    if (q >= ld) return;
    float acc[EG][8];
#pragma unroll
    for (int e = 0; e < EG; ++e)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[e][c] = 0.f;
    const T *x = static_cast<const T *>(a.x) + q;
    for (int bb = 0; bb < a.b; ++bb) {
        float xv[8];
        load8(x + (size_t)bb * ld, xv);
#pragma unroll
        for (int e = 0; e < EG; ++e) {
            const float w = dzs[bb * EG + e];
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[e][c] = fmaf(w, xv[c], acc[e][c]);
        }
    }
    T *dw = static_cast<T *>(a.d_w_e) + q;
#pragma unroll
    for (int e = 0; e < EG; ++e)
        if (e < ne) store8_w<ONCE>(dw + (size_t)(e0 + e) * ld, acc[e]);
}

// d_x[b, q] += sum_i dz[b,i] W_E[i,q]: thread = 8 consecutive q, block.y = a group of 8 samples
template <typename T, bool ONCE> __global__ __launch_bounds__(256) void route_bwd_xexpert_kernel(RouteBwdArgs a)
{
    constexpr int BG = 8;
    __shared__ float dzs[BG * 32];
    const long ld = (long)a.l * a.d, q = ((long)blockIdx.x * 256 + threadIdx.x) * 8;
    const int b0 = blockIdx.y * BG, nb = min(BG, a.b - b0);
    for (int idx = threadIdx.x; idx < BG * a.n; idx += 256) {
        const int s = idx / a.n, i = idx - s * a.n;
        dzs[s * 32 + i] = s < nb ? a.dz[(size_t)(b0 + s) * a.n + i] : 0.f;
    }
    __syncthreads();
    if (q >= ld) return;
    float acc[BG][8];
#pragma unroll
    for (int s = 0; s < BG; ++s)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[s][c] = 0.f;
    const T *w = static_cast<const T *>(a.w_e) + q;
    for (int i = 0; i < a.n; ++i) {
        float wv[8];
        load8_w<ONCE>(w + (size_t)i * ld, wv);
#pragma unroll
        for (int s = 0; s < BG; ++s) {
            const float z = dzs[s * 32 + i];
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[s][c] = fmaf(z, wv[c], acc[s][c]);
        }
    }
    T *dx = static_cast<T *>(a.d_x) + q;
#pragma unroll
    for (int s = 0; s < BG; ++s)
        if (s < nb) {
            float cur[8];
            load8(dx + (size_t)(b0 + s) * ld, cur);
#pragma unroll
            for (int c = 0; c < 8; ++c) cur[c] += acc[s][c];
            store8<T>(dx + (size_t)(b0 + s) * ld, cur);
        }
}

// Data router, per token: U[t,:] = W_A[t,:] dL^T, then one pass over the token's row of x that
// forms (x W_B)[t,:] and adds U[t,:] W_B^T to d_x.  Block = 256/LPT tokens of one sample, LPT lanes
// per token (16 when 4 would leave compute units without a block); the sample's dL and W_B^T
// ([n][d], so that the 8 weights a piece of x meets are one 16-byte read) are staged in LDS.
template <typename T, int LPT> __global__ __launch_bounds__(256) void route_bwd_data_token_kernel(RouteBwdArgs a)
{
    constexpr int TPB = 256 / LPT;  // tokens per block
    extern __shared__ __align__(16) unsigned char smem[];
    float *dls = reinterpret_cast<float *>(smem);                       // [n][m]
    float *us = dls + (size_t)a.n * a.m;                                // [64][n] (TPB <= 64 rows used)
    T *wbt = reinterpret_cast<T *>(smem + ((((size_t)a.n * a.m + 64 * (size_t)a.n) * sizeof(float) + 15) & ~(size_t)15));  // [n][d]
    const int bb = blockIdx.y, tid = threadIdx.x, tl = tid / LPT, part = tid % LPT;
    const int t = blockIdx.x * TPB + tl;
    for (int idx = tid; idx < a.n * a.m; idx += 256) dls[idx] = a.dl[(size_t)bb * a.n * a.m + idx];
    for (int idx = tid; idx < a.d * a.n; idx += 256) {
        const int e = idx / a.n, i = idx - e * a.n;
        wbt[(size_t)i * a.d + e] = static_cast<const T *>(a.w_b)[idx];
    }
    __syncthreads();
    if (t < a.l) {
        const T *wa = static_cast<const T *>(a.w_a) + (size_t)t * a.m;
        for (int i = part; i < a.n; i += LPT) {
            float s = 0.f;
            for (int j = 0; j < a.m; ++j) s = fmaf(to_f32(wa[j]), dls[i * a.m + j], s);
            us[tl * a.n + i] = s;
            a.u[((size_t)bb * a.l + t) * a.n + i] = s;
        }
    }
    __syncthreads();
    float t1[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) t1[i] = 0.f;
    if (t < a.l) {
        const T *xr = static_cast<const T *>(a.x) + ((size_t)bb * a.l + t) * a.d;
        T *dxr = static_cast<T *>(a.d_x) + ((size_t)bb * a.l + t) * a.d;
        for (int pc = part; pc < a.d / 8; pc += LPT) {
            float xv[8], dv[8];
            load8(xr + pc * 8, xv);
            load8(dxr + pc * 8, dv);
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                if (i < a.n) {
                    const float ui = us[tl * a.n + i];
                    float wv[8];
                    load8(wbt + (size_t)i * a.d + pc * 8, wv);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        t1[i] = fmaf(xv[e], wv[e], t1[i]);
                        dv[e] = fmaf(ui, wv[e], dv[e]);
                    }
                }
            }
            store8<T>(dxr + pc * 8, dv);
        }
    }
#pragma unroll
    for (int i = 0; i < 32; ++i)
#pragma unroll
        for (int off = 1; off < LPT; off <<= 1) t1[i] += __shfl_xor(t1[i], off, 64);
    if (t < a.l && part == 0)
        for (int i = 0; i < a.n; ++i) a.t1[((size_t)bb * a.l + t) * a.n + i] = t1[i];
}

// dW_A[t,j] = sum_b sum_i (x W_B)[b,t,i] dL[b,i,j]: thread = (t, j)
template <typename T> __global__ __launch_bounds__(256) void route_bwd_wa_kernel(RouteBwdArgs a)
{
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)a.l * a.m) return;
    const int t = (int)(idx / a.m), j = (int)(idx - (long)t * a.m);
    float s = 0.f;
    for (int bb = 0; bb < a.b; ++bb) {
        const float *t1 = a.t1 + ((size_t)bb * a.l + t) * a.n, *dl = a.dl + (size_t)bb * a.n * a.m + j;
        for (int i = 0; i < a.n; ++i) s = fmaf(t1[i], dl[(size_t)i * a.m], s);
    }
    static_cast<T *>(a.d_w_a)[idx] = from_f32<T>(s);
}

// dW_B[e,i] = sum over all b*l tokens of x[token,e] U[token,i].  Block = a chunk of tokens; thread =
// (8 consecutive e, row lane).  The row lanes' sums are added in lane order through LDS, one
// expert at a time, so that a block leaves one partial [d][n]; the final kernel adds the chunks
// in order.  block.y = a group of 16 experts.
template <typename T> __global__ __launch_bounds__(256) void route_bwd_wb_partial_kernel(RouteBwdArgs a)
{
    constexpr int IG = 16;
    __shared__ float red[256][9];
    __shared__ float us[128 * IG];  // the chunk's rows of U (at most 128 tokens per chunk)
    const int P = a.d / 8, R = 256 / P, tid = threadIdx.x;
    const int pc = tid % P, rl = tid / P;
    const int i0 = blockIdx.y * IG, ni = min(IG, a.n - i0);
    const bool live = rl < R;
    float acc[IG][8];
#pragma unroll
    for (int i = 0; i < IG; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[i][e] = 0.f;
    const long tokens = (long)a.b * a.l, tok0 = (long)blockIdx.x * a.wb_tokens;
    const long tok1 = min(tokens, tok0 + a.wb_tokens);
    const T *x = static_cast<const T *>(a.x);
    const int ntok = (int)(tok1 - tok0);
    for (int idx = tid; idx < ntok * IG; idx += 256) {
        const int tk = idx / IG, i = idx - tk * IG;
        us[idx] = i < ni ? a.u[(tok0 + tk) * a.n + i0 + i] : 0.f;
    }
    __syncthreads();
    if (live) {
        for (int tk = rl; tk < ntok; tk += R) {
            float xv[8];
            load8(x + (tok0 + tk) * a.d + pc * 8, xv);
#pragma unroll
            for (int i = 0; i < IG; ++i) {
                const float ui = us[tk * IG + i];
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[i][e] = fmaf(xv[e], ui, acc[i][e]);
            }
        }
    }
    float *dst = a.wb_part + (size_t)blockIdx.x * a.d * a.n;
#pragma unroll
    for (int i = 0; i < IG; ++i) {  // fully unrolled: acc stays in registers; the skip is uniform
        if (i < ni) {
        if (live)
#pragma unroll
            for (int e = 0; e < 8; ++e) red[tid][e] = acc[i][e];
        __syncthreads();
        if (rl == 0) {
            float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            for (int q = 0; q < R; ++q)
#pragma unroll
                for (int e = 0; e < 8; ++e) s[e] += red[q * P + pc][e];
#pragma unroll
            for (int e = 0; e < 8; ++e) dst[(size_t)(pc * 8 + e) * a.n + i0 + i] = s[e];
        }
        __syncthreads();
        }
    }
}

// adds the chunks' partials in chunk order: block = 32 outputs x 8 part lanes (lane q takes chunks
// q, q+8, ...), then the 8 lanes in lane order
template <typename T> __global__ __launch_bounds__(256) void route_bwd_wb_reduce_kernel(RouteBwdArgs a)
{
    __shared__ float red[8][33];
    const int ol = threadIdx.x & 31, ql = threadIdx.x >> 5;
    const int idx = blockIdx.x * 32 + ol, total = a.d * a.n;
    float s = 0.f;
    if (idx < total)
        for (int p = ql; p < a.wb_chunks; p += 8) s += a.wb_part[(size_t)p * total + idx];
    red[ql][ol] = s;
    __syncthreads();
    if (ql == 0 && idx < total) {
        float v = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) v += red[q][ol];
        static_cast<T *>(a.d_w_b)[idx] = from_f32<T>(v);
    }
}

template <typename T> static hipError_t route_backward(const RouteBwdArgs &a, hipStream_t st)
{
    hipError_t err;
    hipLaunchKernelGGL(route_bwd_softmax_kernel, dim3(a.b, a.w_b ? (a.m + 63) / 64 : 1), dim3(64), 0, st, a);
    if ((err = hipGetLastError()) != hipSuccess) return err;
    const long pieces = (long)a.l * a.d / 8;
    const unsigned pblocks = (unsigned)((pieces + 255) / 256);
    if (a.w_e) {
        const bool once = stream_once((size_t)a.n * a.l * a.d * sizeof(T));
        if (once) hipLaunchKernelGGL((route_bwd_wexpert_kernel<T, true>), dim3(pblocks, (a.n + 7) / 8), dim3(256), 0, st, a);
        else hipLaunchKernelGGL((route_bwd_wexpert_kernel<T, false>), dim3(pblocks, (a.n + 7) / 8), dim3(256), 0, st, a);
        if ((err = hipGetLastError()) != hipSuccess) return err;
        if (once) hipLaunchKernelGGL((route_bwd_xexpert_kernel<T, true>), dim3(pblocks, (a.b + 7) / 8), dim3(256), 0, st, a);
        else hipLaunchKernelGGL((route_bwd_xexpert_kernel<T, false>), dim3(pblocks, (a.b + 7) / 8), dim3(256), 0, st, a);
        if ((err = hipGetLastError()) != hipSuccess) return err;
    }
    if (a.w_b) {
        const size_t smem = ((((size_t)a.n * a.m + 64 * (size_t)a.n) * sizeof(float) + 15) & ~(size_t)15) + (size_t)a.d * a.n * sizeof(T);
        if ((long)((a.l + 63) / 64) * a.b >= 256)
            hipLaunchKernelGGL((route_bwd_data_token_kernel<T, 4>), dim3((a.l + 63) / 64, a.b), dim3(256), smem, st, a);
        else
            hipLaunchKernelGGL((route_bwd_data_token_kernel<T, 16>), dim3((a.l + 15) / 16, a.b), dim3(256), smem, st, a);
        if ((err = hipGetLastError()) != hipSuccess) return err;
        hipLaunchKernelGGL((route_bwd_wa_kernel<T>), dim3((unsigned)(((long)a.l * a.m + 255) / 256)), dim3(256), 0, st, a);
        if ((err = hipGetLastError()) != hipSuccess) return err;
        hipLaunchKernelGGL((route_bwd_wb_partial_kernel<T>), dim3(a.wb_chunks, (a.n + 15) / 16), dim3(256), 0, st, a);
        if ((err = hipGetLastError()) != hipSuccess) return err;
        hipLaunchKernelGGL((route_bwd_wb_reduce_kernel<T>), dim3((a.d * a.n + 31) / 32), dim3(256), 0, st, a);
        if ((err = hipGetLastError()) != hipSuccess) return err;
    }
    return hipSuccess;
}

hipError_t launch_route_backward(const RouteBwdArgs &a, bool bf16, hipStream_t st)
{
    return bf16 ? route_backward<bf16_t>(a, st) : route_backward<float>(a, st);
}

}  // namespace uoe

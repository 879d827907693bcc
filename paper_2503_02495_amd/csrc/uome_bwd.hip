// Backward pass of the expert-selection UoME block (Eq. 38-40 with Eq. 24-26), bf16 storage.
// Forward, per sample b with active experts i(s), s < k, gate w_s (1 without the gate flag):
//   Z = u W1_b           W1_b = [A^I_i(0) | ... | A^I_i(k-1)]            [l, k*d_e]
//   H = SiLU(Z) * w      (column block s scaled by w_s)
//   h = (u) + H W2_b     W2_b = [A^O_i(0); ...; A^O_i(k-1)]              [l, d]
// Backward for an upstream gradient d_out = dL/dh:
//   dH  = d_out W2_b^T                                   GEMM, weights transposed once per call
//   dZ  = dH * w * SiLU'(Z),  H as above,  d_gate[b,i(s)] = sum over block s of dH * SiLU(Z)
//   d_u = (d_out) + dZ W1_b^T                            GEMM
//   dA^O_i = sum_{(b,s): i(s) = i} H_{b,s}^T d_out_b     GEMM over the tokens of those samples
//   dA^I_i = sum_{(b,s): i(s) = i} u_b^T dZ_{b,s}        GEMM over the tokens of those samples
// All five contractions run on the pipelined MFMA engine through the forward problems (the raw
// mode of UomeUpProblem, UomeDownProblem) and WgradProblem; operands the engine wants with K
// contiguous are transposed by a plain tiled copy first (weights: small; u and H: one extra pass
// over the activations).  Z and dH are kept in the storage dtype between the kernels.
#include "common.h"
#include "problems.h"
#include "gemm_mfma.h"
#include "gemm_dma.h"

namespace uoe {

// [batch][rows][cols] -> [batch][cols][rows], 2-byte elements, 32x32 tiles through LDS
__global__ __launch_bounds__(256) void transpose16_kernel(const uint16_t *src, uint16_t *dst, int rows, int cols)
{
    __shared__ uint16_t tile[32][33];
    const size_t base = (size_t)blockIdx.z * rows * cols;
    const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    for (int i = ty; i < 32; i += 8)
        if (r0 + i < rows && c0 + tx < cols) tile[i][tx] = src[base + (size_t)(r0 + i) * cols + c0 + tx];
    __syncthreads();
    for (int i = ty; i < 32; i += 8)
        if (c0 + i < cols && r0 + tx < rows) dst[base + (size_t)(c0 + i) * rows + r0 + tx] = tile[tx][i];
}

static hipError_t launch_transpose(const void *src, void *dst, int batch, int rows, int cols, hipStream_t st)
{
    const dim3 grid((cols + 31) / 32, (rows + 31) / 32, batch);
    hipLaunchKernelGGL(transpose16_kernel, grid, dim3(256), 0, st, static_cast<const uint16_t *>(src),
                       static_cast<uint16_t *>(dst), rows, cols);
    return hipGetLastError();
}

int uome_backward_gate_chunks(int l) { return (l + 63) / 64; }

// Elementwise middle of the backward pass.  Block = (chunk of 64 token rows, slot s, sample b);
// a thread walks 8-element pieces of the slot's d_e columns.  Writes dZ and H, and the block's
// partial sum of dH * SiLU(Z) (summed over the block in a fixed tree, then over chunks by
// uome_bwd_gate_kernel in chunk order).
__global__ __launch_bounds__(256) void uome_bwd_mid_kernel(UomeBwdArgs a)
{
    __shared__ float red[256];
    const int chunk = blockIdx.x, s = blockIdx.y, bb = blockIdx.z, tid = threadIdx.x;
    const int i = clampi(a.expert_idx[bb * a.k + s], a.n);
    const float w = ((a.flags & F_GATE_EXPERT) && a.expert_gate) ? a.expert_gate[(size_t)bb * a.n + i] : 1.0f;
    const int t0 = chunk * 64, rows = min(64, a.l - t0), p8 = a.d_e / 8;
    const size_t width = (size_t)a.k * a.d_e;
    const bf16_t *z = static_cast<const bf16_t *>(a.z), *dh = static_cast<const bf16_t *>(a.dh);
    bf16_t *dz = static_cast<bf16_t *>(a.dz), *h = static_cast<bf16_t *>(a.h);
    float part = 0.f;
    for (int o = tid; o < rows * p8; o += 256) {
        const int r = o / p8, pc = o - r * p8;
        const size_t at = ((size_t)bb * a.l + t0 + r) * width + (size_t)s * a.d_e + pc * 8;
        float zv[8], dv[8];
        load8(z + at, zv);
        load8(dh + at, dv);
        uint32_t oz[4], oh[4];
#pragma unroll
        for (int q = 0; q < 8; q += 2) {
            float dzv[2], hv[2];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const float sig = 1.0f / (1.0f + __expf(-zv[q + e]));
                const float v = zv[q + e] * sig;
                part = fmaf(dv[q + e], v, part);
                hv[e] = v * w;
                dzv[e] = dv[q + e] * w * (sig * (1.0f + zv[q + e] * (1.0f - sig)));
            }
            oz[q / 2] = pack2_bf16(dzv[0], dzv[1]);
            oh[q / 2] = pack2_bf16(hv[0], hv[1]);
        }
        *reinterpret_cast<uint4 *>(dz + at) = make_uint4(oz[0], oz[1], oz[2], oz[3]);
        *reinterpret_cast<uint4 *>(h + at) = make_uint4(oh[0], oh[1], oh[2], oh[3]);
    }
    red[tid] = part;
    __syncthreads();
    for (int st = 128; st > 0; st >>= 1) {
        if (tid < st) red[tid] += red[tid + st];
        __syncthreads();
    }
    if (tid == 0) a.gpart[((size_t)bb * a.k + s) * a.gchunks + chunk] = red[0];
}

// d_gate [b,n]: zero for experts the sample did not select (and everywhere without the gate flag)
__global__ __launch_bounds__(64) void uome_bwd_gate_kernel(UomeBwdArgs a)
{
    const int bb = blockIdx.x, i = threadIdx.x;
    if (i >= a.n) return;
    float v = 0.f;
    if (a.flags & F_GATE_EXPERT)
        for (int s = 0; s < a.k; ++s)
            if (clampi(a.expert_idx[bb * a.k + s], a.n) == i) {
                const float *src = a.gpart + ((size_t)bb * a.k + s) * a.gchunks;
                for (int c = 0; c < a.gchunks; ++c) v += src[c];
                break;
            }
    a.d_gate[(size_t)bb * a.n + i] = v;
}

template <typename P> static hipError_t bwd_gemm(const P &p, int groups, int rows, int ncols, int kseg, hipStream_t st)
{
    const long tiles128 = (long)groups * ((rows + 127) / 128) * ((ncols + 127) / 128);
    if (rows > 128 && (long)groups * ((rows + 255) / 256) * ((ncols + 127) / 128) >= 512)
        return launch_gemm_dma<P, 256, 128, 32, 2, 2, 3, 2>(p, groups, rows, ncols, st);
    if (kseg % 64 == 0 && tiles128 < 256) return launch_gemm_dma<P, 64, 128, 64, 2, 2, 3, 2>(p, groups, rows, ncols, st);
    return kseg % 64 == 0 ? launch_gemm_dma<P, 128, 128, 64, 2, 2, 2, 2>(p, groups, rows, ncols, st)
                          : launch_gemm_dma<P, 128, 128, 32, 2, 2, 4, 2>(p, groups, rows, ncols, st);
}

hipError_t launch_uome_backward(const UomeBwdArgs &a, hipStream_t st)
{
    typedef bf16_t T;
    hipError_t err;
    const int width = a.k * a.d_e;
    // weights with K contiguous for the two data-gradient GEMMs
    if ((err = launch_transpose(a.a_out, a.a_out_t, a.n, a.d_e, a.d, st)) != hipSuccess) return err;  // -> [n, d, d_e]
    if ((err = launch_transpose(a.a_in, a.a_in_t, a.n, a.d, a.d_e, st)) != hipSuccess) return err;    // -> [n, d_e, d]

    UomeUpProblem<T> zp;  // Z = u W1_b
    zp.u = static_cast<const T *>(a.u); zp.a_in = static_cast<const T *>(a.a_in);
    zp.expert_idx = a.expert_idx; zp.expert_gate = nullptr; zp.hidden = static_cast<T *>(a.z);
    zp.l = a.l; zp.d = a.d; zp.n = a.n; zp.kact = a.k; zp.d_e = a.d_e; zp.raw = 1;
    if ((err = bwd_gemm(zp, a.b, a.l, width, a.d, st)) != hipSuccess) return err;
    UomeUpProblem<T> hp = zp;  // dH = d_out W2_b^T: the same contraction with (A^O_i)^T [d, d_e] as the weight
    hp.u = static_cast<const T *>(a.d_out); hp.a_in = static_cast<const T *>(a.a_out_t); hp.hidden = static_cast<T *>(a.dh);
    if ((err = bwd_gemm(hp, a.b, a.l, width, a.d, st)) != hipSuccess) return err;

    hipLaunchKernelGGL(uome_bwd_mid_kernel, dim3(a.gchunks, a.k, a.b), dim3(256), 0, st, a);
    if ((err = hipGetLastError()) != hipSuccess) return err;
    if (a.d_gate) {
        hipLaunchKernelGGL(uome_bwd_gate_kernel, dim3(a.b), dim3(64), 0, st, a);
        if ((err = hipGetLastError()) != hipSuccess) return err;
    }

    UomeDownProblem<T> up;  // d_u = (d_out) + dZ W1_b^T: the second-layer contraction with (A^I_i)^T [d_e, d]
    up.hidden = static_cast<const T *>(a.dz); up.a_out = static_cast<const T *>(a.a_in_t);
    up.u = static_cast<const T *>(a.d_out); up.expert_idx = a.expert_idx; up.out = static_cast<T *>(a.d_u);
    up.l = a.l; up.d = a.d; up.n = a.n; up.kact = a.k; up.d_e = a.d_e; up.flags = a.flags;
    if ((err = bwd_gemm(up, a.b, a.l, a.d, a.d_e, st)) != hipSuccess) return err;

    // weight gradients: left factors with the token axis contiguous
    if ((err = launch_transpose(a.h, a.h_t, a.b, a.l, width, st)) != hipSuccess) return err;  // -> [b, k*d_e, l]
    if ((err = launch_transpose(a.u, a.u_t, a.b, a.l, a.d, st)) != hipSuccess) return err;    // -> [b, d, l]
    WgradProblem<T> wo;  // dA^O_i = sum H_{b,s}^T d_out_b
    wo.left_t = static_cast<const T *>(a.h_t); wo.right = static_cast<const T *>(a.d_out);
    wo.expert_idx = a.expert_idx; wo.dw = static_cast<T *>(a.d_a_out);
    wo.b = a.b; wo.l = a.l; wo.n = a.n; wo.kact = a.k;
    wo.M = a.d_e; wo.N = a.d; wo.left_rows = width; wo.left_slot_rows = a.d_e; wo.right_stride = a.d; wo.right_slot_cols = 0;
    if ((err = bwd_gemm(wo, a.n, a.d_e, a.d, a.l, st)) != hipSuccess) return err;
    WgradProblem<T> wi = wo;  // dA^I_i = sum u_b^T dZ_{b,s}
    wi.left_t = static_cast<const T *>(a.u_t); wi.right = static_cast<const T *>(a.dz); wi.dw = static_cast<T *>(a.d_a_in);
    wi.M = a.d; wi.N = a.d_e; wi.left_rows = a.d; wi.left_slot_rows = 0; wi.right_stride = width; wi.right_slot_cols = a.d_e;
    return bwd_gemm(wi, a.n, a.d, a.d_e, a.l, st);
}

}  // namespace uoe

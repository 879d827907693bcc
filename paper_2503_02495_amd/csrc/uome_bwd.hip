// Backward pass of the UoME block, bf16 storage.  Expert-selection mode first (Eq. 38-40 with
// Eq. 24-26); the data-selection mode (Eq. 37 with Eq. 12-18) follows at the end of the file.
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
// mode of UomeUpProblem, UomeDownProblem) and WgradProblem.  The engine wants every left operand
// K-contiguous: the two weight tensors are transposed by a plain tiled copy (small), the
// elementwise kernel writes H and dZ directly in token-minor layout, and dA^I is formed as its
// transpose (dZ^T u, so that u is the natural-layout right operand) and turned back by the
// reduction that adds the split-K partials.  Z and dH are kept in the storage dtype between the
// kernels.
#include "common.h"
#include "problems.h"
#include "gemm_mfma.h"
#include "gemm_dma.h"
#include "wgrad_reduce.h"

namespace uoe {

// [rows][cols] -> [cols][rows] per expert, 2-byte elements, 32x32 tiles through LDS; both weight
// tensors in one launch
__global__ __launch_bounds__(256) void transpose_weights_kernel(const uint16_t *a_out, uint16_t *a_out_t, const uint16_t *a_in,
                                                                uint16_t *a_in_t, int n, int d, int d_e)
{
    __shared__ uint16_t tile[32][33];
    const bool second = (int)blockIdx.z >= n;
    const int e = second ? blockIdx.z - n : blockIdx.z;
    const int rows = second ? d : d_e, cols = second ? d_e : d;
    const uint16_t *src = (second ? a_in : a_out) + (size_t)e * rows * cols;
    uint16_t *dst = (second ? a_in_t : a_out_t) + (size_t)e * rows * cols;
    const int ctiles = (cols + 31) / 32;
    const int r0 = (blockIdx.x / ctiles) * 32, c0 = (blockIdx.x % ctiles) * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int i = ty; i < 32; i += 8)
        if (r0 + i < rows && c0 + tx < cols) tile[i][tx] = src[(size_t)(r0 + i) * cols + c0 + tx];
    __syncthreads();
    for (int i = ty; i < 32; i += 8)
        if (c0 + i < cols && r0 + tx < rows) dst[(size_t)(c0 + i) * rows + r0 + tx] = tile[tx][i];
}

int uome_backward_gate_chunks(int l, int d_e) { return ((l + 63) / 64) * (d_e / 32); }
int uome_backward_splits(int b, int l, int d, int n, int k, int d_e)
{
    // cut the token axis until the launch has 512 large tiles, while a workgroup keeps on average
    // >= 1024 of K and the ranges stay multiples of 64
    int s = 1;
    const long k_avg = (long)b * k * l / n, tiles = (long)n * ((d_e + 255) / 256) * ((d + 127) / 128);
    while (s < 8 && tiles * s < 512 && l % (2 * s * 64) == 0 && k_avg / (2 * s) >= 1024) s *= 2;
    return s;
}

// Elementwise middle of the backward pass.  Block = (64 token rows, 32 columns of one slot,
// sample b), one 8-element piece per thread.  Writes dZ in token-major layout (the left operand of
// the d_u contraction) and dZ^T, H^T in token-minor layout [b][k*d_e][l] (the left operands of the
// weight gradients) through LDS tiles, and the block's partial sum of dH * SiLU(Z) (fixed tree;
// the partials are then added in index order by uome_bwd_gate_kernel).
__global__ __launch_bounds__(256) void uome_bwd_mid_kernel(UomeBwdArgs a)
{
    constexpr int TP = 72;  // tile pitch in elements: 16-byte aligned rows
    __shared__ float red[256];
    __shared__ __align__(16) uint16_t tz[32][TP], th[32][TP];
    const int chunk = blockIdx.x, cb = blockIdx.y, bb = blockIdx.z, tid = threadIdx.x;
    const int per_slot = a.d_e / 32, s = cb / per_slot;
    const int i = clampi(a.expert_idx[bb * a.k + s], a.n);
    const float w = ((a.flags & F_GATE_EXPERT) && a.expert_gate) ? a.expert_gate[(size_t)bb * a.n + i] : 1.0f;
    const int t0 = chunk * 64, rows = min(64, a.l - t0), c0 = cb * 32;
    const size_t width = (size_t)a.k * a.d_e;
    const bf16_t *z = static_cast<const bf16_t *>(a.z), *dh = static_cast<const bf16_t *>(a.dh);
    bf16_t *dz = static_cast<bf16_t *>(a.dz);
    float part = 0.f;
    {
        const int r = tid >> 2, pc = tid & 3;
        float zv[8] = {0, 0, 0, 0, 0, 0, 0, 0}, dv[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        const size_t at = ((size_t)bb * a.l + t0 + r) * width + c0 + pc * 8;
        if (r < rows) {
            load8(z + at, zv);
            load8(dh + at, dv);
        }
        uint32_t oz[4];
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
            const uint32_t oh = pack2_bf16(hv[0], hv[1]);
            tz[pc * 8 + q][r] = (uint16_t)(oz[q / 2] & 0xFFFFu);
            tz[pc * 8 + q + 1][r] = (uint16_t)(oz[q / 2] >> 16);
            th[pc * 8 + q][r] = (uint16_t)(oh & 0xFFFFu);
            th[pc * 8 + q + 1][r] = (uint16_t)(oh >> 16);
        }
        if (r < rows) *reinterpret_cast<uint4 *>(dz + at) = make_uint4(oz[0], oz[1], oz[2], oz[3]);
    }
    red[tid] = part;
    __syncthreads();
    {
        const int col = tid >> 3, tp = tid & 7;  // 8 consecutive tokens of one column
        if (tp * 8 < rows) {
            const size_t at = ((size_t)bb * width + c0 + col) * a.l + t0 + tp * 8;
            *reinterpret_cast<uint4 *>(static_cast<bf16_t *>(a.dz_t) + at) = *reinterpret_cast<const uint4 *>(&tz[col][tp * 8]);
            *reinterpret_cast<uint4 *>(static_cast<bf16_t *>(a.h_t) + at) = *reinterpret_cast<const uint4 *>(&th[col][tp * 8]);
        }
    }
    for (int st = 128; st > 0; st >>= 1) {
        if (tid < st) red[tid] += red[tid + st];
        __syncthreads();
    }
    if (tid == 0) a.gpart[((size_t)bb * a.k + s) * a.gchunks + chunk * per_slot + (cb - s * per_slot)] = red[0];
}

// d_gate [b,n]: block (slot s, sample b) adds the slot's partial sums (each thread a strided
// subset in index order, then a fixed tree) into the entry of the slot's expert; the block of slot 0
// also writes the zeros of the experts the sample did not select (all of them without the gate flag).
__global__ __launch_bounds__(256) void uome_bwd_gate_kernel(UomeBwdArgs a)
{
    __shared__ float red[256];
    const int s = blockIdx.x, bb = blockIdx.y, tid = threadIdx.x;
    const bool gated = a.flags & F_GATE_EXPERT;
    if (s == 0 && tid < a.n) {
        bool chosen = false;
        for (int q = 0; q < a.k; ++q) chosen |= clampi(a.expert_idx[bb * a.k + q], a.n) == tid;
        if (!chosen || !gated) a.d_gate[(size_t)bb * a.n + tid] = 0.f;
    }
    if (!gated) return;
    const float *src = a.gpart + ((size_t)bb * a.k + s) * a.gchunks;
    float v = 0.f;
    for (int c = tid; c < a.gchunks; c += 256) v += src[c];
    red[tid] = v;
    __syncthreads();
    for (int st = 128; st > 0; st >>= 1) {
        if (tid < st) red[tid] += red[tid + st];
        __syncthreads();
    }
    if (tid == 0) a.d_gate[(size_t)bb * a.n + clampi(a.expert_idx[bb * a.k + s], a.n)] = red[0];
}

hipError_t launch_uome_ds_backward(const UomeBwdArgs &a, hipStream_t st);

hipError_t launch_uome_backward(const UomeBwdArgs &a, hipStream_t st)
{
    typedef bf16_t T;
    if (a.patch_idx) return launch_uome_ds_backward(a, st);
    hipError_t err;
    const int width = a.k * a.d_e;
    // weights with K contiguous for the two data-gradient GEMMs
    {   // one launch: blocks z < n take A^O [d_e, d] -> [d, d_e], the others A^I [d, d_e] -> [d_e, d]
        const int tiles = ((a.d + 31) / 32) * ((a.d_e + 31) / 32);
        hipLaunchKernelGGL(transpose_weights_kernel, dim3(tiles, 1, 2 * a.n), dim3(256), 0, st,
                           static_cast<const uint16_t *>(a.a_out), static_cast<uint16_t *>(a.a_out_t),
                           static_cast<const uint16_t *>(a.a_in), static_cast<uint16_t *>(a.a_in_t), a.n, a.d, a.d_e);
        if ((err = hipGetLastError()) != hipSuccess) return err;
    }

    UomeUpProblem<T, true> zp;  // Z = u W1_b (plain product)
    zp.u = static_cast<const T *>(a.u); zp.a_in = static_cast<const T *>(a.a_in);
    zp.expert_idx = a.expert_idx; zp.expert_gate = nullptr; zp.hidden = static_cast<T *>(a.z);
    zp.l = a.l; zp.d = a.d; zp.n = a.n; zp.kact = a.k; zp.d_e = a.d_e;
    zp.once = stream_once((size_t)a.b * a.l * width * sizeof(T));   // Z and dH: written here, read once by the next kernel
    if ((err = launch_gemm_dma_auto(zp, a.b, a.l, width, a.d, st)) != hipSuccess) return err;
    UomeUpProblem<T, true> hp = zp;  // dH = d_out W2_b^T: the same contraction with (A^O_i)^T [d, d_e] as the weight
    hp.u = static_cast<const T *>(a.d_out); hp.a_in = static_cast<const T *>(a.a_out_t); hp.hidden = static_cast<T *>(a.dh);
    if ((err = launch_gemm_dma_auto(hp, a.b, a.l, width, a.d, st)) != hipSuccess) return err;

    hipLaunchKernelGGL(uome_bwd_mid_kernel, dim3((a.l + 63) / 64, width / 32, a.b), dim3(256), 0, st, a);
    if ((err = hipGetLastError()) != hipSuccess) return err;
    if (a.d_gate) {
        hipLaunchKernelGGL(uome_bwd_gate_kernel, dim3(a.k, a.b), dim3(256), 0, st, a);
        if ((err = hipGetLastError()) != hipSuccess) return err;
    }

    UomeDownProblem<T> up;  // d_u = (d_out) + dZ W1_b^T: the second-layer contraction with (A^I_i)^T [d_e, d]
    up.hidden = static_cast<const T *>(a.dz); up.a_out = static_cast<const T *>(a.a_in_t);
    up.u = static_cast<const T *>(a.d_out); up.expert_idx = a.expert_idx; up.out = static_cast<T *>(a.d_u);
    up.l = a.l; up.d = a.d; up.n = a.n; up.kact = a.k; up.d_e = a.d_e; up.flags = a.flags;
    if ((err = launch_gemm_dma_auto(up, a.b, a.l, a.d, a.d_e, st)) != hipSuccess) return err;

    // weight gradients, both in one launch: [d_e, d] tiles per expert, token axis cut into a.splits
    // ranges; (dA^I_i)^T = sum dZ_{b,s}^T u_b is stored back as [d, d_e] by the reduction
    WgradProblem<T> wp;
    wp.left_t[0] = static_cast<const T *>(a.h_t); wp.right[0] = static_cast<const T *>(a.d_out);  // dA^O_i
    wp.left_t[1] = static_cast<const T *>(a.dz_t); wp.right[1] = static_cast<const T *>(a.u);     // (dA^I_i)^T
    wp.expert_idx = a.expert_idx; wp.partial = a.partial;
    wp.b = a.b; wp.l = a.l; wp.n = a.n; wp.kact = a.k; wp.splits = a.splits;
    wp.M = a.d_e; wp.N = a.d; wp.left_rows = width; wp.left_slot_rows = a.d_e; wp.right_stride = a.d;
    if ((err = launch_gemm_dma_auto(wp, 2 * a.n * a.splits, a.d_e, a.d, a.l / a.splits, st)) != hipSuccess) return err;
    WgradReduceArgs ra{};
    ra.partial = a.partial; ra.n = a.n; ra.M = a.d_e; ra.N = a.d; ra.splits = a.splits;
    ra.dst[0] = static_cast<uint16_t *>(a.d_a_out); ra.transposed[0] = 0;
    ra.dst[1] = static_cast<uint16_t *>(a.d_a_in); ra.transposed[1] = 1;
    return launch_wgrad_reduce(ra, 2, st);
}

// ---------------------------------------------------------------------------------------------
// Data-selection mode (Eq. 37-40 with Eq. 12-18): expert i of an active unit sees only the l_a
// gathered rows of its c patches.  Same chain as above per unit, with the gathers folded into
// operand addressing (the forward's gathered projection for Z and dH, the output-stationary
// per-patch contraction for d_u, patch-gathered right operands for the weight gradients) and the
// row weight w_t = expert gate and/or the gate of the row's patch.

// Elementwise middle, data-selection mode.  Block = 32 rows of one unit; it walks the d_e columns in
// tiles of 64 (one 8-element piece per thread and tile), writes dZ token-major, dZ^T and H^T
// token-minor through LDS tiles, and the rows' dL/dw_t = sum_j dH_raw * SiLU(Z).
__global__ __launch_bounds__(256) void uome_ds_bwd_mid_kernel(UomeBwdArgs a)
{
    __shared__ __align__(16) uint16_t tz[64][40], th[64][40];
    const int g = blockIdx.y, tid = threadIdx.x, r = tid >> 3, pc = tid & 7;
    const int l_p = a.l / a.m, l_a = a.c * l_p, row = blockIdx.x * 32 + r;
    const int bb = g / a.k, i = clampi(a.expert_idx[g], a.n);
    float w = 1.0f;
    if ((a.flags & F_GATE_EXPERT) && a.expert_gate) w *= a.expert_gate[(size_t)bb * a.n + i];
    if ((a.flags & F_GATE_PATCH) && a.patch_gate) {
        const int p = clampi(a.patch_idx[((size_t)bb * a.n + i) * a.c + row / l_p], a.m);
        w *= a.patch_gate[((size_t)bb * a.n + i) * a.m + p];
    }
    const bf16_t *z = static_cast<const bf16_t *>(a.z), *dh = static_cast<const bf16_t *>(a.dh);
    bf16_t *dz = static_cast<bf16_t *>(a.dz);
    float part = 0.f;
    for (int c0 = 0; c0 < a.d_e; c0 += 64) {
        const int col = c0 + pc * 8;
        float zv[8] = {0, 0, 0, 0, 0, 0, 0, 0}, dv[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        const size_t at = ((size_t)g * l_a + row) * a.d_e + col;
        if (col < a.d_e) {
            load8(z + at, zv);
            load8(dh + at, dv);
        }
        uint32_t oz[4];
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
            const uint32_t oh = pack2_bf16(hv[0], hv[1]);
            tz[pc * 8 + q][r] = (uint16_t)(oz[q / 2] & 0xFFFFu);
            tz[pc * 8 + q + 1][r] = (uint16_t)(oz[q / 2] >> 16);
            th[pc * 8 + q][r] = (uint16_t)(oh & 0xFFFFu);
            th[pc * 8 + q + 1][r] = (uint16_t)(oh >> 16);
        }
        if (col < a.d_e) *reinterpret_cast<uint4 *>(dz + at) = make_uint4(oz[0], oz[1], oz[2], oz[3]);
        __syncthreads();
        const int tc = tid >> 2, tp = tid & 3;  // column of the tile, 8 consecutive rows
        if (c0 + tc < a.d_e) {
            const size_t to = ((size_t)g * a.d_e + c0 + tc) * l_a + blockIdx.x * 32 + tp * 8;
            *reinterpret_cast<uint4 *>(static_cast<bf16_t *>(a.dz_t) + to) = *reinterpret_cast<const uint4 *>(&tz[tc][tp * 8]);
            *reinterpret_cast<uint4 *>(static_cast<bf16_t *>(a.h_t) + to) = *reinterpret_cast<const uint4 *>(&th[tc][tp * 8]);
        }
        __syncthreads();
    }
    part += __shfl_xor(part, 1, 64);
    part += __shfl_xor(part, 2, 64);
    part += __shfl_xor(part, 4, 64);
    if (pc == 0) a.rt[(size_t)g * l_a + row] = part;
}

hipError_t launch_uome_ds_backward(const UomeBwdArgs &a, hipStream_t st)
{
    typedef bf16_t T;
    hipError_t err;
    const int l_p = a.l / a.m, l_a = a.c * l_p, units = a.b * a.k;
    {
        const int tiles = ((a.d + 31) / 32) * ((a.d_e + 31) / 32);
        hipLaunchKernelGGL(transpose_weights_kernel, dim3(tiles, 1, 2 * a.n), dim3(256), 0, st,
                           static_cast<const uint16_t *>(a.a_out), static_cast<uint16_t *>(a.a_out_t),
                           static_cast<const uint16_t *>(a.a_in), static_cast<uint16_t *>(a.a_in_t), a.n, a.d, a.d_e);
        if ((err = hipGetLastError()) != hipSuccess) return err;
    }
    // Z = u[T] A^I_i and dH_raw = d_out[T] A^O_i^T: the gathered projection with one output block
    QkvProblem<T> zp;
    zp.x = static_cast<const T *>(a.u);
    zp.wq = zp.wk = zp.wv = static_cast<const T *>(a.a_in);
    zp.expert_idx = a.expert_idx; zp.patch_idx = a.patch_idx;
    zp.q = zp.k = zp.v = static_cast<T *>(a.z); zp.q32 = nullptr;
    zp.l = a.l; zp.d = a.d; zp.n = a.n; zp.kact = a.k; zp.m = a.m; zp.c = a.c;
    zp.l_p = l_p; zp.l_a = l_a; zp.d_h = a.d_e; zp.q_scale = 1.0f; zp.nout = 1;
    if ((err = launch_gemm_dma_auto(zp, units, l_a, a.d_e, a.d, st)) != hipSuccess) return err;
    QkvProblem<T> hp = zp;
    hp.x = static_cast<const T *>(a.d_out);
    hp.wq = hp.wk = hp.wv = static_cast<const T *>(a.a_out_t);
    hp.q = hp.k = hp.v = static_cast<T *>(a.dh);
    if ((err = launch_gemm_dma_auto(hp, units, l_a, a.d_e, a.d, st)) != hipSuccess) return err;

    hipLaunchKernelGGL(uome_ds_bwd_mid_kernel, dim3(l_a / 32, units), dim3(256), 0, st, a);
    if ((err = hipGetLastError()) != hipSuccess) return err;

    SmhaBwdArgs ga{};  // the unit gate kernel reads its routing fields, the row terms and the gates
    ga.f.expert_idx = a.expert_idx; ga.f.patch_idx = a.patch_idx;
    ga.f.b = a.b; ga.f.l = a.l; ga.f.d = a.d; ga.f.n = a.n; ga.f.k = a.k; ga.f.m = a.m; ga.f.c = a.c;
    ga.expert_gate = a.expert_gate; ga.patch_gate = a.patch_gate; ga.flags = a.flags;
    ga.d_expert_gate = a.d_gate; ga.d_patch_gate = a.d_patch_gate; ga.rt = a.rt;
    if ((err = launch_unit_gate_grads(ga, st)) != hipSuccess) return err;

    // d_u = (d_out) + scatter-add of dZ A^I_i^T: the output-stationary per-patch contraction
    OutProjProblem<T> xp;
    xp.o = static_cast<const T *>(a.dz); xp.o_lo = nullptr; xp.parts = 1;
    xp.wo = static_cast<const T *>(a.a_in_t); xp.x = static_cast<const T *>(a.d_out);
    xp.expert_idx = a.expert_idx; xp.patch_idx = a.patch_idx; xp.inv_cnt = nullptr; xp.inv_ent = nullptr;
    xp.out = static_cast<T *>(a.d_u);
    xp.l = a.l; xp.d = a.d; xp.n = a.n; xp.kact = a.k; xp.m = a.m; xp.c = a.c;
    xp.l_p = l_p; xp.l_a = l_a; xp.d_h = a.d_e; xp.flags = a.flags & F_RESIDUAL;
    if (l_p <= 32) err = launch_gemm_dma<OutProjProblem<T>, 32, 128, 32, 1, 4, 4, 2>(xp, a.b * a.m, l_p, a.d, st);
    else err = launch_gemm_dma<OutProjProblem<T>, 64, 128, 32, 2, 2, 4, 2>(xp, a.b * a.m, l_p, a.d, st);
    if (err != hipSuccess) return err;

    SmhaWgradProblem<T> wp;  // both weight gradients in one launch
    wp.left_t[0] = static_cast<const T *>(a.h_t); wp.right[0] = static_cast<const T *>(a.d_out);  // dA^O_i
    wp.left_t[1] = static_cast<const T *>(a.dz_t); wp.right[1] = static_cast<const T *>(a.u);     // (dA^I_i)^T
    wp.left_t[2] = wp.left_t[3] = wp.right[2] = wp.right[3] = nullptr;
    for (int q = 0; q < 4; ++q) { wp.unit_rows[q] = a.d_e; wp.row0[q] = 0; }
    wp.expert_idx = a.expert_idx; wp.patch_idx = a.patch_idx; wp.partial = a.partial;
    wp.b = a.b; wp.l = a.l; wp.d = a.d; wp.n = a.n; wp.kact = a.k; wp.m = a.m; wp.c = a.c;
    wp.l_p = l_p; wp.l_a = l_a; wp.splits = a.splits; wp.M = a.d_e;
    if ((err = launch_gemm_dma_auto(wp, 2 * a.n * a.splits, a.d_e, a.d, l_p, st)) != hipSuccess) return err;
    WgradReduceArgs ra{};
    ra.partial = a.partial; ra.n = a.n; ra.M = a.d_e; ra.N = a.d; ra.splits = a.splits;
    ra.dst[0] = static_cast<uint16_t *>(a.d_a_out); ra.transposed[0] = 0;
    ra.dst[1] = static_cast<uint16_t *>(a.d_a_in); ra.transposed[1] = 1;
    return launch_wgrad_reduce(ra, 2, st);
}

}  // namespace uoe

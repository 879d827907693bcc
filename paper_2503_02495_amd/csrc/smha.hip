// Selective Multi-Head Attention on given routing results (Eq. 27-36).
//
// Pipeline per call (all on one stream):
//   smha_inverse_map : for each (sample, patch) the list of (active slot s, pick t) that chose
//                      it -- the transpose of patch_idx restricted to active experts.
//   QKV projection   : grouped GEMM over active units, Eq. 18 gather folded into the A rows.
//   attention        : softmax(q k^T / sqrt(d_h)) v per unit over its l_a tokens (Eq. 33-34),
//                      rows scaled by their gate weight on the way out.
//   out-projection   : output-stationary grouped GEMM over (sample, patch) that concatenates the
//                      contributions of every expert that picked the patch along K and writes
//                      each output row once, residual included (Eq. 35-36).
#include "common.h"
#include "problems.h"
#include "gemm_generic.h"
#include "gemm_mfma.h"

namespace uoe {

// one thread per (sample, patch); picks of an expert are ascending so a linear scan suffices
__global__ __launch_bounds__(256) void smha_inverse_map_kernel(SmhaArgs a)
{
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= a.b * a.m) return;
    const int bb = g / a.m, p = g - bb * a.m;
    int cnt = 0;
    for (int s = 0; s < a.k; ++s) {
        const int i = clampi(a.expert_idx[bb * a.k + s], a.n);
        const int32_t *pid = a.patch_idx + ((size_t)bb * a.n + i) * a.c;
        for (int t = 0; t < a.c; ++t)
            if (pid[t] == p) {
                a.inv_ent[(size_t)g * a.k + cnt] = s * a.c + t;
                ++cnt;
                break;
            }
    }
    a.inv_cnt[g] = cnt;
}

// Vector-ALU attention: one thread per query row, keys/values staged through LDS in tiles,
// online softmax in fp32.  DH is d_h rounded up to a supported register-array size.
template <typename T, int DH>
__global__ __launch_bounds__(128) void attention_generic_kernel(SmhaArgs a)
{
    constexpr int KT = 32;  // keys per LDS tile
    __shared__ float ks[KT][DH + 1];
    __shared__ float vs[KT][DH + 1];
    const int g = blockIdx.y;  // unit
    const int l_p = a.l / a.m, l_a = a.c * l_p, d_h = a.d_h;
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    const bool live = r < l_a;
    const T *q = static_cast<const T *>(a.q) + (size_t)g * l_a * d_h;
    const T *kp = static_cast<const T *>(a.kk) + (size_t)g * l_a * d_h;
    const T *vp = static_cast<const T *>(a.v) + (size_t)g * l_a * d_h;
    const float scale = rsqrtf((float)d_h);

    float qr[DH], acc[DH];
#pragma unroll
    for (int e = 0; e < DH; ++e) {
        qr[e] = (live && e < d_h) ? to_f32(q[(size_t)r * d_h + e]) * scale : 0.f;
        acc[e] = 0.f;
    }
    float mx = -INFINITY, den = 0.f;

    for (int j0 = 0; j0 < l_a; j0 += KT) {
        const int jn = min(KT, l_a - j0);
        for (int idx = threadIdx.x; idx < KT * DH; idx += blockDim.x) {
            const int jj = idx / DH, e = idx - jj * DH;
            const bool ok = jj < jn && e < d_h;
            ks[jj][e] = ok ? to_f32(kp[(size_t)(j0 + jj) * d_h + e]) : 0.f;
            vs[jj][e] = ok ? to_f32(vp[(size_t)(j0 + jj) * d_h + e]) : 0.f;
        }
        __syncthreads();
        if (live) {
            for (int jj = 0; jj < jn; ++jj) {
                float s = 0.f;
#pragma unroll
                for (int e = 0; e < DH; ++e) s = fmaf(qr[e], ks[jj][e], s);
                const float nmx = fmaxf(mx, s);
                const float corr = __expf(mx - nmx);  // exp(-inf) = 0 on the first key
                const float pw = __expf(s - nmx);
                den = den * corr + pw;
#pragma unroll
                for (int e = 0; e < DH; ++e) acc[e] = fmaf(acc[e], corr, pw * vs[jj][e]);
                mx = nmx;
            }
        }
        __syncthreads();
    }
    if (!live) return;
    // gate weight of this row (Eq. 36 with the optional gate flags)
    const int bb = g / a.k, i = clampi(a.expert_idx[g], a.n);
    float w = 1.0f;
    if ((a.flags & F_GATE_EXPERT) && a.expert_gate) w *= a.expert_gate[(size_t)bb * a.n + i];
    if ((a.flags & F_GATE_PATCH) && a.patch_gate) {
        const int p = clampi(a.patch_idx[((size_t)bb * a.n + i) * a.c + r / l_p], a.m);
        w *= a.patch_gate[((size_t)bb * a.n + i) * a.m + p];
    }
    const float inv = w / den;
    T *o = static_cast<T *>(a.o) + ((size_t)g * l_a + r) * d_h;
#pragma unroll
    for (int e = 0; e < DH; ++e)
        if (e < d_h) o[e] = from_f32<T>(acc[e] * inv);
}

template <typename T> static hipError_t launch_attention_generic(const SmhaArgs &a, hipStream_t st)
{
    const int l_a = a.c * (a.l / a.m);
    dim3 grid((l_a + 127) / 128, a.b * a.k), block(128);
    if (a.d_h <= 16) hipLaunchKernelGGL((attention_generic_kernel<T, 16>), grid, block, 0, st, a);
    else if (a.d_h <= 32) hipLaunchKernelGGL((attention_generic_kernel<T, 32>), grid, block, 0, st, a);
    else if (a.d_h <= 64) hipLaunchKernelGGL((attention_generic_kernel<T, 64>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((attention_generic_kernel<T, 128>), grid, block, 0, st, a);
    return hipGetLastError();
}

template <typename T> static QkvProblem<T> make_qkv(const SmhaArgs &a)
{
    QkvProblem<T> qp;
    qp.x = static_cast<const T *>(a.x);
    qp.wq = static_cast<const T *>(a.wq);
    qp.wk = static_cast<const T *>(a.wk);
    qp.wv = static_cast<const T *>(a.wv);
    qp.expert_idx = a.expert_idx;
    qp.patch_idx = a.patch_idx;
    qp.q = static_cast<T *>(a.q);
    qp.k = static_cast<T *>(a.kk);
    qp.v = static_cast<T *>(a.v);
    qp.l = a.l; qp.d = a.d; qp.n = a.n; qp.kact = a.k; qp.m = a.m; qp.c = a.c;
    qp.l_p = a.l / a.m; qp.l_a = a.c * qp.l_p; qp.d_h = a.d_h;
    qp.v_transposed = 0; qp.l_a_pad = qp.l_a; qp.q_scale = 1.0f;
    return qp;
}

template <typename T> static OutProjProblem<T> make_outproj(const SmhaArgs &a)
{
    OutProjProblem<T> op;
    op.o = static_cast<const T *>(a.o);
    op.wo = static_cast<const T *>(a.wo);
    op.x = static_cast<const T *>(a.x);
    op.expert_idx = a.expert_idx;
    op.inv_cnt = a.inv_cnt;
    op.inv_ent = a.inv_ent;
    op.out = static_cast<T *>(a.out);
    op.l = a.l; op.d = a.d; op.n = a.n; op.kact = a.k; op.m = a.m; op.c = a.c;
    op.l_p = a.l / a.m; op.l_a = a.c * op.l_p; op.d_h = a.d_h; op.flags = a.flags;
    return op;
}

template <typename T> static hipError_t smha_generic(const SmhaArgs &a, hipStream_t st)
{
    const int l_p = a.l / a.m, l_a = a.c * l_p, units = a.b * a.k;
    hipError_t err;
    hipLaunchKernelGGL(smha_inverse_map_kernel, dim3((a.b * a.m + 255) / 256), dim3(256), 0, st, a);
    if ((err = hipGetLastError()) != hipSuccess) return err;
    if ((err = launch_gemm_generic<T>(make_qkv<T>(a), units, l_a, 3 * a.d_h, st)) != hipSuccess) return err;
    if ((err = launch_attention_generic<T>(a, st)) != hipSuccess) return err;
    return launch_gemm_generic<T>(make_outproj<T>(a), a.b * a.m, l_p, a.d, st);
}

// MFMA path: bf16 storage, d and d_h multiples of 32 (the K segments of the two projections)
static hipError_t smha_mfma(const SmhaArgs &a, hipStream_t st)
{
    typedef QkvProblem<bf16_t> QP;
    typedef OutProjProblem<bf16_t> OP;
    const int l_p = a.l / a.m, l_a = a.c * l_p, units = a.b * a.k;
    hipError_t err;
    hipLaunchKernelGGL(smha_inverse_map_kernel, dim3((a.b * a.m + 255) / 256), dim3(256), 0, st, a);
    if ((err = hipGetLastError()) != hipSuccess) return err;

    const QP qp = make_qkv<bf16_t>(a);
    // one workgroup row-tile computes q, k and v together so the gathered rows are read once
    if (a.d_h == 32) err = launch_gemm_mfma<QP, 128, 96, 4, 1>(qp, units, l_a, 96, st);
    else if (a.d_h == 64) err = launch_gemm_mfma<QP, 128, 192, 4, 1>(qp, units, l_a, 192, st);
    else err = launch_gemm_mfma<QP, 128, 128, 2, 2>(qp, units, l_a, 3 * a.d_h, st);
    if (err != hipSuccess) return err;

    if ((err = launch_attention_generic<bf16_t>(a, st)) != hipSuccess) return err;

    const OP op = make_outproj<bf16_t>(a);
    if (l_p <= 32) return launch_gemm_mfma<OP, 32, 128, 1, 4>(op, a.b * a.m, l_p, a.d, st);
    return launch_gemm_mfma<OP, 64, 128, 2, 2>(op, a.b * a.m, l_p, a.d, st);
}

hipError_t launch_smha(const SmhaArgs &a, bool bf16, hipStream_t st)
{
    if (bf16 && a.d % 32 == 0 && a.d_h % 32 == 0) return smha_mfma(a, st);
    return bf16 ? smha_generic<bf16_t>(a, st) : smha_generic<float>(a, st);
}

}  // namespace uoe

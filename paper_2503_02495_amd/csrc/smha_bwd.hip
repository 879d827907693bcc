// Backward pass of the SMHA block (Eq. 27-36 with the partial RoPE of Eq. 32 and the masks of
// Sec. III-C.3), bf16 storage, MFMA shapes.  For an upstream gradient G = dL/du [b,l,d], per active unit (sample b,
// slot s, expert i) with gathered token positions T, gate weight w_t of row t (Eq. 36 with the
// gate flags), o = softmax(q k^T / sqrt(d_h)) v and y = o W^O_i (u[T_t] += w_t y_t):
//   dO_raw = G[T] W^O_i^T,   r_t = dO_raw_t . o_t  (= dL/dw_t),   dO = w * dO_raw
//   dW^O_i += (w * o)^T G[T]
//   d_expert_gate[b,i] = sum_t g_patch(t) r_t,  d_patch_gate[b,i,p] = g_expert * sum_{t in p} r_t
//   P = softmax(...), dV = P^T dO, dP = dO V^T, dS = P * (dP - D) with D_i = sum_j P_ij dP_ij,
//   dQ = dS K / sqrt(d_h), dK = dS^T Q / sqrt(d_h)  (both rotated back when q, k were rotated)
//   dW^{q,k,v}_i += x[T]^T d{Q,K,V},   d_x[T] += dQ W^q_i^T + dK W^k_i^T + dV W^v_i^T  (+ G: residual)
// The forward intermediates are recomputed with the forward's own kernels (projections and
// attention, which also keeps each query's log-sum-exp); the contractions with the weights run on
// the pipelined GEMM engine (gathers folded into operand addressing as in the forward pass; the
// scatter-add of d_x output-stationary per patch, no atomics); the attention backward is a pair of
// MFMA kernels (one owning query rows, one owning key rows) that never materialise P.
#include "common.h"
#include "problems.h"
#include "gemm_mfma.h"
#include "gemm_dma.h"
#include "wgrad_reduce.h"

namespace uoe {

// Set-up in one launch.  Blocks z < 4n transpose one 32x32 tile of a weight (2-byte elements):
// job 0 turns W^O_i [d_h, d] into [d, d_h]; jobs 1-3 turn W^q_i, W^k_i, W^v_i [d, d_h] into row
// blocks of [3*d_h, d].  Blocks z == 4n clear the two gate-gradient outputs.
struct SmhaBwdPrepArgs {
    const uint16_t *w[4];  // wo, wq, wk, wv
    uint16_t *wo_t, *wqkv_t;
    float *zero[2];
    long zero_count[2];
    int n, d, d_h;
};

__global__ __launch_bounds__(256) void smha_bwd_prep_kernel(SmhaBwdPrepArgs a)
{
    __shared__ uint16_t tile[32][33];
    const int z = blockIdx.z;
    if (z == 4 * a.n) {
        const long at = ((long)blockIdx.y * gridDim.x + blockIdx.x) * 256 + threadIdx.x, step = (long)gridDim.x * gridDim.y * 256;
        for (int q = 0; q < 2; ++q)
            if (a.zero[q])
                for (long i = at; i < a.zero_count[q]; i += step) a.zero[q][i] = 0.f;
        return;
    }
    const int job = z / a.n, e = z - job * a.n;
    const int rows = job == 0 ? a.d_h : a.d, cols = job == 0 ? a.d : a.d_h;
    // the grid covers the larger of the two tile counts in each direction
    const int r0 = (job == 0 ? blockIdx.x : blockIdx.y) * 32, c0 = (job == 0 ? blockIdx.y : blockIdx.x) * 32;
    if (r0 >= rows || c0 >= cols) return;
    const uint16_t *src = a.w[job] + (size_t)e * a.d * a.d_h;
    uint16_t *dst = job == 0 ? a.wo_t + (size_t)e * a.d * a.d_h
                             : a.wqkv_t + (size_t)e * 3 * a.d * a.d_h + (size_t)(job - 1) * a.d * a.d_h;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int i = ty; i < 32; i += 8)
        if (r0 + i < rows && c0 + tx < cols) tile[i][tx] = src[(size_t)(r0 + i) * cols + c0 + tx];
    __syncthreads();
    for (int i = ty; i < 32; i += 8)
        if (c0 + i < cols && r0 + tx < rows) dst[(size_t)(c0 + i) * rows + r0 + tx] = tile[tx][i];
}

// Row pass between the out-projection gradient and the attention gradient.  Block = 32 rows of one
// unit, thread = one 8-element piece of a row.  r_t (fp32), dO = w * dO_raw (token-major, rounded
// once from the fp32 product), (w * o)^T (token-minor, through an LDS tile).
template <int DH> __global__ __launch_bounds__(4 * DH) void smha_bwd_row_kernel(SmhaBwdArgs a)
{
    constexpr int PPR = DH / 8;  // pieces (= threads) per row
    __shared__ __align__(16) uint16_t tl[DH][40];
    const int g = blockIdx.y, tid = threadIdx.x;
    const int l_p = a.f.l / a.f.m, l_a = a.f.c * l_p;
    const int r = tid / PPR, pc = tid % PPR, row = blockIdx.x * 32 + r;
    const int bb = g / a.f.k, i = clampi(a.f.expert_idx[g], a.f.n);
    float w = 1.0f;
    if (a.flags & F_GATE_EXPERT) w *= a.expert_gate[(size_t)bb * a.f.n + i];
    if (a.flags & F_GATE_PATCH) {
        const int p = clampi(a.f.patch_idx[((size_t)bb * a.f.n + i) * a.f.c + row / l_p], a.f.m);
        w *= a.patch_gate[((size_t)bb * a.f.n + i) * a.f.m + p];
    }
    const size_t at = ((size_t)g * l_a + row) * DH + pc * 8;
    float dor[8], oh[8], ol[8];
    load8(a.do_raw + at, dor);
    load8(static_cast<const bf16_t *>(a.f.o) + at, oh);
    load8(static_cast<const bf16_t *>(a.f.o_lo) + at, ol);
    float dot = 0.f;
    uint32_t od[4];
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
        const float o0 = oh[e] + ol[e], o1 = oh[e + 1] + ol[e + 1];
        dot = fmaf(dor[e], o0, dot);
        dot = fmaf(dor[e + 1], o1, dot);
        od[e / 2] = pack2_bf16(dor[e] * w, dor[e + 1] * w);
        const uint32_t og = pack2_bf16(o0 * w, o1 * w);
        tl[pc * 8 + e][r] = (uint16_t)(og & 0xFFFFu);
        tl[pc * 8 + e + 1][r] = (uint16_t)(og >> 16);
    }
    *reinterpret_cast<uint4 *>(static_cast<bf16_t *>(a.d_o) + at) = make_uint4(od[0], od[1], od[2], od[3]);
#pragma unroll
    for (int off = PPR / 2; off >= 1; off >>= 1) dot += __shfl_xor(dot, off, 64);
    if (pc == 0) a.rt[(size_t)g * l_a + row] = dot;
    __syncthreads();
    const int col = tid >> 2, tp = tid & 3;
    *reinterpret_cast<uint4 *>(static_cast<bf16_t *>(a.o_t) + ((size_t)g * DH + col) * l_a + blockIdx.x * 32 + tp * 8) =
        *reinterpret_cast<const uint4 *>(&tl[col][tp * 8]);
}

// Gate gradients of one unit from the row sums r_t: wave w takes picks w, w+4, ...; the pick sums
// are then combined in pick order.  The outputs were zero-filled before.
__global__ __launch_bounds__(256) void smha_bwd_gate_kernel(SmhaBwdArgs a)
{
    __shared__ float ps[1024];
    const int g = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l_p = a.f.l / a.f.m, l_a = a.f.c * l_p;
    const int bb = g / a.f.k, i = clampi(a.f.expert_idx[g], a.f.n);
    const float *rt = a.rt + (size_t)g * l_a;
    for (int t = wave; t < a.f.c; t += 4) {
        float v = 0.f;
        for (int q = lane; q < l_p; q += 64) v += rt[t * l_p + q];
        v = wave_sum(v);
        if (lane == 0) ps[t] = v;
    }
    __syncthreads();
    const int32_t *pid = a.f.patch_idx + ((size_t)bb * a.f.n + i) * a.f.c;
    const float *gp = (a.flags & F_GATE_PATCH) ? a.patch_gate + ((size_t)bb * a.f.n + i) * a.f.m : nullptr;
    if ((a.flags & F_GATE_PATCH) && a.d_patch_gate) {
        const float ge = (a.flags & F_GATE_EXPERT) ? a.expert_gate[(size_t)bb * a.f.n + i] : 1.0f;
        for (int t = tid; t < a.f.c; t += 256) a.d_patch_gate[((size_t)bb * a.f.n + i) * a.f.m + clampi(pid[t], a.f.m)] = ge * ps[t];
    }
    if ((a.flags & F_GATE_EXPERT) && a.d_expert_gate && tid == 0) {
        float v = 0.f;
        for (int t = 0; t < a.f.c; ++t) v += (gp ? gp[clampi(pid[t], a.f.m)] : 1.0f) * ps[t];
        a.d_expert_gate[(size_t)bb * a.f.n + i] = v;
    }
}

// ---------------------------------------------------------------------------------------------
// Attention backward.  One wave owns 32 rows of one unit ("own" rows) and walks the unit's other
// axis in tiles of 64 ("streamed" rows): KV = false owns queries and streams keys (dQ), KV = true
// owns keys and streams queries (dK, dV).  Everything is computed transposed, as in the forward
// kernel, so that an accumulator lane holds one own row:
//   S^T [streamed x own] = TA fa^T,  dP^T = TB fb^T      (TA/TB streamed tiles, fa/fb own fragments)
//   P^T = exp2(S^T - lse[query]),  dS^T = P^T * (dP^T - D[query]),  D[i] = sum_j P_ij dP_ij
//   accA^T [d_h x own] += TA^T dS^T        (dQ = K^T-contraction; dK = Q^T-contraction)
//   accB^T [d_h x own] += TB^T P^T         (KV only: dV = dO^T-contraction)
// with (TA, TB, fa, fb) = (k, v, q, dO) for KV = false and (q, dO, k, v) for KV = true.  q arrives
// scaled by log2(e)/sqrt(d_h) (base-2 softmax), so dK = ln 2 * accA and dQ = accA / sqrt(d_h).
// P^T and dS^T, rounded to bf16 in place, are the B operands of the second products; the A
// operands come out of the [row][d_h] LDS tiles through the transposing read.  Outputs go to the
// [dq | dk | dv] buffer in token-major layout (left operand of the d_x contraction) and in
// token-minor layout (left operand of the weight gradients).
struct AttnBwdArgs {
    const bf16_t *q, *k, *v, *d_o;
    const float *lse;
    float *dd;              // [units, l_a]: written by the query-owning kernel, read by the key-owning one
    bf16_t *dqkv, *dqkv_t;  // [units, l_a, 3*d_h], [units, 3*d_h, l_a]
    int l_a, causal;
    int rope_dim;           // Eq. 32: dq and dk are rotated back (the transposed rotation) on the way out
    // Eq. 41: padded keys are out of every softmax.  pad_mask [b,l] (1 = token) or NULL, looked up
    // through the unit's patch indices
    const unsigned char *pad_mask;
    const int32_t *expert_idx, *patch_idx;
    int l, n, kact, c, m, l_p;
};

__device__ __forceinline__ bool bwd_key_is_token(const AttnBwdArgs &a, int g, int key)
{
    const int bb = g / a.kact, i = clampi(a.expert_idx[g], a.n);
    const int p = clampi(a.patch_idx[((size_t)bb * a.n + i) * a.c + key / a.l_p], a.m);
    return a.pad_mask[(size_t)bb * a.l + p * a.l_p + key % a.l_p] != 0;
}

template <int DH, int NW, bool KV, bool PAD> __global__ __launch_bounds__(NW * 64) void attention_bwd_kernel(AttnBwdArgs a)
{
    constexpr int BT = 64, KP = DH + 8, VP = 2 * b_pitch_dwords(DH), NT = NW * 64;
    constexpr int CHUNKS = BT * DH / 8, PER_T = (CHUNKS + NT - 1) / NT;
    __shared__ __align__(16) uint16_t TAr[BT][KP];
    __shared__ __align__(16) uint16_t TAt[BT][VP];
    __shared__ __align__(16) uint16_t TBr[BT][KP];
    __shared__ __align__(16) uint16_t TBt[KV ? BT : 1][VP];
    __shared__ __align__(16) float Ls[BT], Ds[BT];
    __shared__ unsigned char Km[PAD ? BT : 1];  // streamed key admissible under the padding mask (KV = false)

    const int g = blockIdx.y, l_a = a.l_a;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lr = lane & 31, lh = lane >> 5;
    const int orow = blockIdx.x * (32 * NW) + wave * 32 + lr;
    const size_t ubase = (size_t)g * l_a * DH;
    const bf16_t *own_a = (KV ? a.k : a.q) + ubase, *own_b = (KV ? a.v : a.d_o) + ubase;
    const bf16_t *str_a = (KV ? a.q : a.k) + ubase, *str_b = (KV ? a.d_o : a.v) + ubase;

    bf16x8_t fa[DH / 16], fb[DH / 16];
#pragma unroll
    for (int ks = 0; ks < DH / 16; ++ks) {
        uint4 va = make_uint4(0, 0, 0, 0), vb = make_uint4(0, 0, 0, 0);
        if (orow < l_a) {
            va = *reinterpret_cast<const uint4 *>(own_a + (size_t)orow * DH + ks * 16 + lh * 8);
            vb = *reinterpret_cast<const uint4 *>(own_b + (size_t)orow * DH + ks * 16 + lh * 8);
        }
        fa[ks] = __builtin_bit_cast(bf16x8_t, va);
        fb[ks] = __builtin_bit_cast(bf16x8_t, vb);
    }
    float lse_o = 0.f, d_own = 0.f;
    if (!KV && orow < l_a) lse_o = a.lse[(size_t)g * l_a + orow];
    constexpr bool padded = PAD;  // compile-time: the unmasked kernels keep two waves per SIMD
    const bool own_key_ok = !(KV && padded) || bwd_key_is_token(a, g, min(orow, l_a - 1));

    f32x16_t acc_a[DH / 32], acc_b[DH / 32];
#pragma unroll
    for (int t = 0; t < DH / 32; ++t)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc_a[t][q] = acc_b[t][q] = 0.f;

    // streamed tiles: under the causal mask a query sees keys <= itself
    const int blk0 = blockIdx.x * 32 * NW, blk1 = min(l_a, blk0 + 32 * NW);
    int t_begin = 0, t_end = (l_a + BT - 1) / BT;
    if (a.causal) {
        if (KV) t_begin = blk0 / BT;
        else t_end = (blk1 + BT - 1) / BT;
    }

    uint4 ra[PER_T], rb[PER_T];
    float lreg = 0.f, dreg = 0.f;
    unsigned char kmreg = 1;
    auto load_global = [&](int row0) {
#pragma unroll
        for (int i = 0; i < PER_T; ++i) {
            const int c = tid + i * NT;
            const int row = c / (DH / 8), kc = c % (DH / 8);
            uint4 va = make_uint4(0, 0, 0, 0), vb = make_uint4(0, 0, 0, 0);
            if (c < CHUNKS && row0 + row < l_a) {
                va = *reinterpret_cast<const uint4 *>(str_a + (size_t)(row0 + row) * DH + kc * 8);
                vb = *reinterpret_cast<const uint4 *>(str_b + (size_t)(row0 + row) * DH + kc * 8);
            }
            ra[i] = va;
            rb[i] = vb;
        }
        if (KV && tid < BT) {
            const bool in = row0 + tid < l_a;
            lreg = in ? a.lse[(size_t)g * l_a + row0 + tid] : 0.f;
            dreg = in ? a.dd[(size_t)g * l_a + row0 + tid] : 0.f;
        }
        if (!KV && padded && tid < BT) kmreg = row0 + tid < l_a && bwd_key_is_token(a, g, min(row0 + tid, l_a - 1));
    };
    auto store_lds = [&]() {
#pragma unroll
        for (int i = 0; i < PER_T; ++i) {
            const int c = tid + i * NT;
            if (c < CHUNKS) {
                const int row = c / (DH / 8), col = (c % (DH / 8)) * 8;
                *reinterpret_cast<uint4 *>(&TAr[row][col]) = ra[i];
                *reinterpret_cast<uint4 *>(&TAt[row][col]) = ra[i];
                *reinterpret_cast<uint4 *>(&TBr[row][col]) = rb[i];
                if (KV) *reinterpret_cast<uint4 *>(&TBt[row][col]) = rb[i];
            }
        }
        if (KV && tid < BT) {
            Ls[tid] = lreg;
            Ds[tid] = dreg;
        }
        if (!KV && padded && tid < BT) Km[tid] = kmreg;
    };

    // first products of one tile and the probabilities: leaves P^T in sacc and dP^T in pacc
    auto scores = [&](int kt, f32x16_t (&sacc)[2], f32x16_t (&pacc)[2]) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int q = 0; q < 16; ++q) sacc[t][q] = pacc[t][q] = 0.f;
#pragma unroll
        for (int ks = 0; ks < DH / 16; ++ks)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const bf16x8_t ta = *reinterpret_cast<const bf16x8_t *>(&TAr[t * 32 + lr][ks * 16 + lh * 8]);
                sacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ta, fa[ks], sacc[t], 0, 0, 0);
                const bf16x8_t tb = *reinterpret_cast<const bf16x8_t *>(&TBr[t * 32 + lr][ks * 16 + lh * 8]);
                pacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tb, fb[ks], pacc[t], 0, 0, 0);
            }
        // accumulator register q of tile t is streamed row kt*64 + t*32 + (q/4)*8 + lh*4 + q%4
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int qg = 0; qg < 4; ++qg) {
                const int cl0 = t * 32 + qg * 8 + lh * 4;
                float l4[4] = {lse_o, lse_o, lse_o, lse_o};
                if (KV) {
                    const float4 lv = *reinterpret_cast<const float4 *>(&Ls[cl0]);
                    l4[0] = lv.x; l4[1] = lv.y; l4[2] = lv.z; l4[3] = lv.w;
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int q = qg * 4 + e, crow = kt * BT + cl0 + e;
                    const int query = KV ? crow : orow, key = KV ? orow : crow;
                    const float p = __builtin_amdgcn_exp2f(sacc[t][q] - l4[e]);
                    bool key_ok = true;
                    if constexpr (PAD) key_ok = KV ? own_key_ok : Km[cl0 + e] != 0;
                    sacc[t][q] = (crow >= l_a || (a.causal && key > query) || !key_ok) ? 0.f : p;
                }
            }
    };

    // Owning the queries, a first walk over the keys forms the softmax row term from the very
    // values the second walk uses, D = sum_j P_ij dP_ij, so that the rows of dS cancel to zero
    // as they do in exact arithmetic (a row that attends to one key gets dS = 0, not the rounding
    // difference of two separately rounded numbers); it is kept for the key-owning kernel.
    if (!KV) {
        float dsum = 0.f;
        if (t_begin < t_end) load_global(t_begin * BT);
        for (int kt = t_begin; kt < t_end; ++kt) {
            __syncthreads();
            store_lds();
            __syncthreads();
            if (kt + 1 < t_end) load_global((kt + 1) * BT);
            f32x16_t sacc[2], pacc[2];
            scores(kt, sacc, pacc);
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int q = 0; q < 16; ++q) dsum = fmaf(sacc[t][q], pacc[t][q], dsum);
        }
        dsum += __shfl_xor(dsum, 32, 64);
        d_own = dsum;
        if (orow < l_a && lh == 0) a.dd[(size_t)g * l_a + orow] = dsum;
    }

    if (t_begin < t_end) load_global(t_begin * BT);
    for (int kt = t_begin; kt < t_end; ++kt) {
        __syncthreads();  // the previous tile has been consumed
        store_lds();
        __syncthreads();
        if (kt + 1 < t_end) load_global((kt + 1) * BT);

        f32x16_t sacc[2], pacc[2];
        scores(kt, sacc, pacc);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int qg = 0; qg < 4; ++qg) {
                float d4[4] = {d_own, d_own, d_own, d_own};
                if (KV) {
                    const float4 dv = *reinterpret_cast<const float4 *>(&Ds[t * 32 + qg * 8 + lh * 4]);
                    d4[0] = dv.x; d4[1] = dv.y; d4[2] = dv.z; d4[3] = dv.w;
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) pacc[t][qg * 4 + e] = sacc[t][qg * 4 + e] * (pacc[t][qg * 4 + e] - d4[e]);
            }
        // second products over the 64 streamed rows: four k-steps of 16; dS^T and P^T enter as
        // (hi, lo) bf16 pairs, which keeps ~16 of their bits
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
            const int t = s4 >> 1, r0 = (s4 & 1) * 8;
            uint32_t dsh[4], dsl[4], ph[4], pl[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float x0 = pacc[t][r0 + 2 * e], x1 = pacc[t][r0 + 2 * e + 1];
                dsh[e] = pack2_bf16(x0, x1);
                dsl[e] = pack2_bf16(x0 - __uint_as_float(dsh[e] << 16), x1 - __uint_as_float(dsh[e] & 0xFFFF0000u));
                if (KV) {
                    const float p0 = sacc[t][r0 + 2 * e], p1 = sacc[t][r0 + 2 * e + 1];
                    ph[e] = pack2_bf16(p0, p1);
                    pl[e] = pack2_bf16(p0 - __uint_as_float(ph[e] << 16), p1 - __uint_as_float(ph[e] & 0xFFFF0000u));
                }
            }
            const bf16x8_t ds_hi = __builtin_bit_cast(bf16x8_t, make_uint4(dsh[0], dsh[1], dsh[2], dsh[3]));
            const bf16x8_t ds_lo = __builtin_bit_cast(bf16x8_t, make_uint4(dsl[0], dsl[1], dsl[2], dsl[3]));
            const int trow = s4 * 16 + lh * 4 + ((lane & 15) >> 2);
#pragma unroll
            for (int td = 0; td < DH / 32; ++td) {
                const int tcol = td * 32 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
                const uint2 a0 = lds_read_tr4(&TAt[trow][tcol]);
                const uint2 a1 = lds_read_tr4(&TAt[trow + 8][tcol]);
                const bf16x8_t taf = __builtin_bit_cast(bf16x8_t, make_uint4(a0.x, a0.y, a1.x, a1.y));
                acc_a[td] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(taf, ds_hi, acc_a[td], 0, 0, 0);
                acc_a[td] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(taf, ds_lo, acc_a[td], 0, 0, 0);
                if (KV) {
                    const bf16x8_t p_hi = __builtin_bit_cast(bf16x8_t, make_uint4(ph[0], ph[1], ph[2], ph[3]));
                    const bf16x8_t p_lo = __builtin_bit_cast(bf16x8_t, make_uint4(pl[0], pl[1], pl[2], pl[3]));
                    const uint2 b0 = lds_read_tr4(&TBt[trow][tcol]);
                    const uint2 b1 = lds_read_tr4(&TBt[trow + 8][tcol]);
                    const bf16x8_t tbf = __builtin_bit_cast(bf16x8_t, make_uint4(b0.x, b0.y, b1.x, b1.y));
                    acc_b[td] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tbf, p_hi, acc_b[td], 0, 0, 0);
                    acc_b[td] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tbf, p_lo, acc_b[td], 0, 0, 0);
                }
            }
        }
    }

    if (orow >= l_a) return;
    // accumulator register q of tile td is head-dim index td*32 + (q/4)*8 + lh*4 + q%4
    const float scale_a = KV ? 0.6931471805599453f : rsqrtf((float)DH);
    bf16_t *row_out = a.dqkv + ((size_t)g * l_a + orow) * (3 * DH);
    bf16_t *col_out = a.dqkv_t + (size_t)g * (3 * DH) * l_a + orow;
    // q and k were rotated in adjacent pairs (2i, 2i+1) of the last rope_dim dims, row r by r * theta_i;
    // the gradient of the unrotated projection is the gradient rotated by -r * theta_i.  A lane's four
    // consecutive head dims hold two whole pairs (rope_dim and d_h are even).
    const int rope_first = DH - a.rope_dim;
    auto put = [&](const f32x16_t (&acc)[DH / 32], int block, float scale) {
#pragma unroll
        for (int td = 0; td < DH / 32; ++td)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int dh0 = td * 32 + i4 * 8 + lh * 4;
                float v[4] = {acc[td][i4 * 4 + 0] * scale, acc[td][i4 * 4 + 1] * scale, acc[td][i4 * 4 + 2] * scale,
                              acc[td][i4 * 4 + 3] * scale};
                if (block < 2 && a.rope_dim > 0) {
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const int dh = dh0 + 2 * h;
                        if (dh >= rope_first) {
                            const float theta = exp2f(-((float)(dh - rope_first) / (float)a.rope_dim) * 13.287712379549449f);
                            float sn, cs;
                            sincosf((float)orow * theta, &sn, &cs);
                            const float ga = v[2 * h], gb = v[2 * h + 1];
                            v[2 * h] = ga * cs + gb * sn;
                            v[2 * h + 1] = gb * cs - ga * sn;
                        }
                    }
                }
                const uint32_t w0 = pack2_bf16(v[0], v[1]);
                const uint32_t w1 = pack2_bf16(v[2], v[3]);
                *reinterpret_cast<uint2 *>(row_out + block * DH + dh0) = make_uint2(w0, w1);
                uint16_t *ct = reinterpret_cast<uint16_t *>(col_out) + (size_t)(block * DH + dh0) * l_a;
                ct[0] = (uint16_t)(w0 & 0xFFFFu);
                ct[l_a] = (uint16_t)(w0 >> 16);
                ct[2 * (size_t)l_a] = (uint16_t)(w1 & 0xFFFFu);
                ct[3 * (size_t)l_a] = (uint16_t)(w1 >> 16);
            }
    };
    if (KV) {
        put(acc_a, 1, scale_a);
        put(acc_b, 2, 1.0f);
    } else {
        put(acc_a, 0, scale_a);
    }
}

template <int DH, bool PAD> static hipError_t launch_attention_bwd_dh(const AttnBwdArgs &a, int units, hipStream_t st)
{
    const int l_a = a.l_a;
    if ((long)((l_a + 127) / 128) * units >= 128) {
        const dim3 grid((l_a + 127) / 128, units);
        hipLaunchKernelGGL((attention_bwd_kernel<DH, 4, false, PAD>), grid, dim3(256), 0, st, a);
        hipLaunchKernelGGL((attention_bwd_kernel<DH, 4, true, PAD>), grid, dim3(256), 0, st, a);
    } else if ((long)((l_a + 63) / 64) * units >= 64) {
        const dim3 grid((l_a + 63) / 64, units);
        hipLaunchKernelGGL((attention_bwd_kernel<DH, 2, false, PAD>), grid, dim3(128), 0, st, a);
        hipLaunchKernelGGL((attention_bwd_kernel<DH, 2, true, PAD>), grid, dim3(128), 0, st, a);
    } else {
        const dim3 grid((l_a + 31) / 32, units);
        hipLaunchKernelGGL((attention_bwd_kernel<DH, 1, false, PAD>), grid, dim3(64), 0, st, a);
        hipLaunchKernelGGL((attention_bwd_kernel<DH, 1, true, PAD>), grid, dim3(64), 0, st, a);
    }
    return hipGetLastError();
}

template <bool PAD> static hipError_t launch_attention_bwd(const AttnBwdArgs &a, int dh, int units, hipStream_t st)
{
    if (dh == 32) return launch_attention_bwd_dh<32, PAD>(a, units, st);
    if (dh == 64) return launch_attention_bwd_dh<64, PAD>(a, units, st);
    return launch_attention_bwd_dh<128, PAD>(a, units, st);
}

hipError_t launch_unit_gate_grads(const SmhaBwdArgs &a, hipStream_t st)
{
    const SmhaArgs &f = a.f;
    SmhaBwdPrepArgs pa{};  // only its clearing blocks run: n = 0 puts them at z = 0
    pa.zero[0] = a.d_expert_gate; pa.zero_count[0] = (long)f.b * f.n;
    pa.zero[1] = a.d_patch_gate; pa.zero_count[1] = (long)f.b * f.n * f.m;
    pa.n = 0; pa.d = f.d; pa.d_h = 32;
    hipLaunchKernelGGL(smha_bwd_prep_kernel, dim3(8, 8, 1), dim3(256), 0, st, pa);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    if (a.flags & (F_GATE_EXPERT | F_GATE_PATCH)) {
        hipLaunchKernelGGL(smha_bwd_gate_kernel, dim3(f.b * f.k), dim3(256), 0, st, a);
        err = hipGetLastError();
    }
    return err;
}

int smha_backward_splits(int b, int n, int k, int c)
{
    // parts of an expert's (unit, pick) list: about 8 segments each, at most 8 parts, and never more
    // than 128 segments in one part even if every sample selected the expert
    const int avg = (int)(((long)b * k * c + n - 1) / n);
    int s = avg / 8;
    s = s < 1 ? 1 : (s > 8 ? 8 : s);
    const int need = (b * c + 127) / 128;
    return s > need ? s : need;
}

hipError_t launch_smha_backward(const SmhaBwdArgs &a, hipStream_t st)
{
    typedef bf16_t T;
    const SmhaArgs &f = a.f;
    const int l_p = f.l / f.m, l_a = f.c * l_p, units = f.b * f.k, dh = f.d_h;
    hipError_t err;

    {   // weights with K contiguous, cleared gate outputs
        SmhaBwdPrepArgs pa;
        pa.w[0] = static_cast<const uint16_t *>(f.wo); pa.w[1] = static_cast<const uint16_t *>(f.wq);
        pa.w[2] = static_cast<const uint16_t *>(f.wk); pa.w[3] = static_cast<const uint16_t *>(f.wv);
        pa.wo_t = static_cast<uint16_t *>(a.wo_t); pa.wqkv_t = static_cast<uint16_t *>(a.wqkv_t);
        pa.zero[0] = a.d_expert_gate; pa.zero_count[0] = (long)f.b * f.n;
        pa.zero[1] = a.d_patch_gate; pa.zero_count[1] = (long)f.b * f.n * f.m;
        pa.n = f.n; pa.d = f.d; pa.d_h = dh;
        hipLaunchKernelGGL(smha_bwd_prep_kernel, dim3((dh + 31) / 32, (f.d + 31) / 32, 4 * f.n + 1), dim3(256), 0, st, pa);
        if ((err = hipGetLastError()) != hipSuccess) return err;
    }

    // forward intermediates: q (scaled for the base-2 softmax), k, v, ungated o = hi + lo, lse
    if ((err = launch_smha_qkv_attention(f, st)) != hipSuccess) return err;

    // dO_raw = G[T] W^O^T: the forward's gathered projection with one output block
    QkvProblem<T, true> dp;
    dp.x = static_cast<const T *>(a.d_out);
    dp.wq = dp.wk = dp.wv = static_cast<const T *>(a.wo_t);
    dp.expert_idx = f.expert_idx; dp.patch_idx = f.patch_idx;
    dp.q = dp.k = dp.v = nullptr;
    dp.q32 = a.do_raw;
    dp.l = f.l; dp.d = f.d; dp.n = f.n; dp.kact = f.k; dp.m = f.m; dp.c = f.c;
    dp.l_p = l_p; dp.l_a = l_a; dp.d_h = dh; dp.q_scale = 1.0f; dp.nout = 1;
    if ((err = launch_gemm_dma_auto(dp, units, l_a, dh, f.d, st)) != hipSuccess) return err;

    const dim3 rgrid(l_a / 32, units);
    if (dh == 32) hipLaunchKernelGGL((smha_bwd_row_kernel<32>), rgrid, dim3(128), 0, st, a);
    else if (dh == 64) hipLaunchKernelGGL((smha_bwd_row_kernel<64>), rgrid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((smha_bwd_row_kernel<128>), rgrid, dim3(512), 0, st, a);
    if ((err = hipGetLastError()) != hipSuccess) return err;
    if (a.flags & (F_GATE_EXPERT | F_GATE_PATCH)) {
        hipLaunchKernelGGL(smha_bwd_gate_kernel, dim3(units), dim3(256), 0, st, a);
        if ((err = hipGetLastError()) != hipSuccess) return err;
    }

    AttnBwdArgs ab;
    ab.q = static_cast<const T *>(f.q); ab.k = static_cast<const T *>(f.kk); ab.v = static_cast<const T *>(f.v);
    ab.d_o = static_cast<const T *>(a.d_o); ab.lse = f.lse; ab.dd = a.dd;
    ab.dqkv = static_cast<T *>(a.dqkv); ab.dqkv_t = static_cast<T *>(a.dqkv_t);
    ab.l_a = l_a; ab.causal = (f.flags & F_CAUSAL) ? 1 : 0; ab.rope_dim = f.rope_dim;
    ab.pad_mask = f.pad_mask; ab.expert_idx = f.expert_idx; ab.patch_idx = f.patch_idx;
    ab.l = f.l; ab.n = f.n; ab.kact = f.k; ab.c = f.c; ab.m = f.m; ab.l_p = l_p;
    err = ab.pad_mask ? launch_attention_bwd<true>(ab, dh, units, st) : launch_attention_bwd<false>(ab, dh, units, st);
    if (err != hipSuccess) return err;

    // d_x = (G) + scatter-add of [dq|dk|dv] [W^q|W^k|W^v]^T: the out-projection's output-stationary
    // contraction with 3*d_h as the expert's K segment
    OutProjProblem<T> xp;
    xp.o = static_cast<const T *>(a.dqkv); xp.o_lo = nullptr; xp.parts = 1;
    xp.wo = static_cast<const T *>(a.wqkv_t); xp.x = static_cast<const T *>(a.d_out);
    xp.expert_idx = f.expert_idx; xp.patch_idx = f.patch_idx; xp.inv_cnt = nullptr; xp.inv_ent = nullptr;
    xp.out = static_cast<T *>(a.d_x);
    xp.l = f.l; xp.d = f.d; xp.n = f.n; xp.kact = f.k; xp.m = f.m; xp.c = f.c;
    xp.l_p = l_p; xp.l_a = l_a; xp.d_h = 3 * dh; xp.flags = a.flags & F_RESIDUAL;
    if (l_p <= 32) err = launch_gemm_dma<OutProjProblem<T>, 32, 128, 32, 1, 4, 4, 2>(xp, f.b * f.m, l_p, f.d, st);
    else err = launch_gemm_dma<OutProjProblem<T>, 64, 128, 32, 2, 2, 4, 2>(xp, f.b * f.m, l_p, f.d, st);
    if (err != hipSuccess) return err;

    // weight gradients, all four in one launch (M = d_h each): sets 0-2 = (dW^q, dW^k, dW^v)^T from
    // the rows of [dq|dk|dv]^T against gathered x, set 3 = dW^O from (w*o)^T against gathered d_out
    SmhaWgradProblem<T> wp;
    for (int q = 0; q < 3; ++q) {
        wp.left_t[q] = static_cast<const T *>(a.dqkv_t); wp.right[q] = static_cast<const T *>(f.x);
        wp.unit_rows[q] = 3 * dh; wp.row0[q] = q * dh;
    }
    wp.left_t[3] = static_cast<const T *>(a.o_t); wp.right[3] = static_cast<const T *>(a.d_out);
    wp.unit_rows[3] = dh; wp.row0[3] = 0;
    wp.expert_idx = f.expert_idx; wp.patch_idx = f.patch_idx; wp.partial = a.partial;
    wp.b = f.b; wp.l = f.l; wp.d = f.d; wp.n = f.n; wp.kact = f.k; wp.m = f.m; wp.c = f.c;
    wp.l_p = l_p; wp.l_a = l_a; wp.splits = a.splits; wp.M = dh;
    if ((err = launch_gemm_dma_auto(wp, 4 * f.n * a.splits, dh, f.d, l_p, st)) != hipSuccess) return err;
    WgradReduceArgs ra{};
    ra.partial = a.partial; ra.n = f.n; ra.M = dh; ra.N = f.d; ra.splits = a.splits;
    ra.dst[0] = static_cast<uint16_t *>(a.d_wq); ra.dst[1] = static_cast<uint16_t *>(a.d_wk);
    ra.dst[2] = static_cast<uint16_t *>(a.d_wv); ra.dst[3] = static_cast<uint16_t *>(a.d_wo);
    ra.transposed[0] = ra.transposed[1] = ra.transposed[2] = 1; ra.transposed[3] = 0;
    return launch_wgrad_reduce(ra, 4, st);
}

}  // namespace uoe

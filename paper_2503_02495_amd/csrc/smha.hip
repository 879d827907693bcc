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
#include "gemm_dma.h"

namespace uoe {

// Inverse map, one workgroup per sample.  Phase 1: one thread per (active slot s, pick t) writes
// t into an LDS table slot_of[s][patch].  Phase 2: one thread per patch walks the k slots in
// order and lists the (s, t) pairs that chose it, so the list order (and with it the summation
// order of the out-projection) is fixed.
__global__ __launch_bounds__(256) void smha_inverse_map_kernel(SmhaArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    int16_t *slot_of = reinterpret_cast<int16_t *>(smem);  // [k][m], -1 = not picked
    const int bb = blockIdx.x, tid = threadIdx.x;
    const int km = a.k * a.m, kc = a.k * a.c;
    for (int idx = tid; idx < km; idx += 256) slot_of[idx] = -1;
    __syncthreads();
    for (int idx = tid; idx < kc; idx += 256) {
        const int s = idx / a.c, t = idx - s * a.c;
        const int i = clampi(a.expert_idx[bb * a.k + s], a.n);
        const int p = clampi(a.patch_idx[((size_t)bb * a.n + i) * a.c + t], a.m);
        slot_of[s * a.m + p] = (int16_t)t;
    }
    __syncthreads();
    for (int p = tid; p < a.m; p += 256) {
        const size_t g = (size_t)bb * a.m + p;
        int cnt = 0;
        for (int s = 0; s < a.k; ++s) {
            const int t = slot_of[s * a.m + p];
            if (t >= 0) a.inv_ent[g * a.k + cnt++] = s * a.c + t;
        }
        a.inv_cnt[g] = cnt;
    }
}

static hipError_t launch_inverse_map(const SmhaArgs &a, hipStream_t st)
{
    const size_t sh = (size_t)a.k * a.m * sizeof(int16_t);  // <= 32 * 1024 * 2 = 64 KiB
    hipLaunchKernelGGL(smha_inverse_map_kernel, dim3(a.b), dim3(256), sh, st, a);
    return hipGetLastError();
}

// Partial RoPE of Eq. 32, in place on the q and k workspaces: the last rope_dim dims of a head are
// rotated in adjacent pairs (2i, 2i+1) by position * 10000^(-2i/rope_dim); the position of a row
// is its index in the unit's compacted sequence.  One thread per (unit row, pair).
template <typename T> __global__ __launch_bounds__(256) void smha_rope_kernel(SmhaArgs a)
{
    const int l_a = a.c * (a.l / a.m), half = a.rope_dim >> 1;
    const long total = (long)a.b * a.k * l_a * half;
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int i = (int)(idx % half);
    const long row = idx / half;              // unit * l_a + r
    const int r = (int)(row % l_a);
    const float theta = exp2f(-(2.0f * (float)i / (float)a.rope_dim) * 13.287712379549449f);  // log2(10000)
    float sn, cs;
    sincosf((float)r * theta, &sn, &cs);
    const size_t at = (size_t)row * a.d_h + (a.d_h - a.rope_dim) + 2 * i;
    T *q = static_cast<T *>(a.q) + at, *k = static_cast<T *>(a.kk) + at;
    const float q0 = to_f32(q[0]), q1 = to_f32(q[1]), k0 = to_f32(k[0]), k1 = to_f32(k[1]);
    q[0] = from_f32<T>(q0 * cs - q1 * sn);
    q[1] = from_f32<T>(q0 * sn + q1 * cs);
    k[0] = from_f32<T>(k0 * cs - k1 * sn);
    k[1] = from_f32<T>(k0 * sn + k1 * cs);
}

template <typename T> static hipError_t launch_rope(const SmhaArgs &a, hipStream_t st)
{
    if (a.rope_dim <= 0) return hipSuccess;
    const long total = (long)a.b * a.k * a.c * (a.l / a.m) * (a.rope_dim >> 1);
    hipLaunchKernelGGL((smha_rope_kernel<T>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, a);
    return hipGetLastError();
}

// padding flag of key `key` of unit g (Eq. 41: the mask is gathered with the unit's indices)
__device__ __forceinline__ bool key_is_token(const SmhaArgs &a, int g, int key, int l_p)
{
    const int bb = g / a.k, i = clampi(a.expert_idx[g], a.n);
    const int p = clampi(a.patch_idx[((size_t)bb * a.n + i) * a.c + key / l_p], a.m);
    return a.pad_mask[(size_t)bb * a.l + p * l_p + key % l_p] != 0;
}

// Vector-ALU attention: one thread per query row, keys/values staged through LDS in tiles,
// online softmax in fp32.  DH is d_h rounded up to a supported register-array size.
template <typename T, int DH>
__global__ __launch_bounds__(128) void attention_generic_kernel(SmhaArgs a)
{
    constexpr int KT = 32;  // keys per LDS tile
    __shared__ float ks[KT][DH + 1];
    __shared__ float vs[KT][DH + 1];
    __shared__ unsigned char km[KT];  // key admissible under the padding mask
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
    const bool causal = (a.flags & F_CAUSAL) != 0;
    // under the causal mask no row of this block sees keys past the block's last row
    const int key_end = causal ? min(l_a, (int)((blockIdx.x + 1) * blockDim.x)) : l_a;

    for (int j0 = 0; j0 < key_end; j0 += KT) {
        const int jn = min(KT, l_a - j0);
        if (threadIdx.x < KT)
            km[threadIdx.x] = (threadIdx.x < jn) && (!a.pad_mask || key_is_token(a, g, j0 + threadIdx.x, l_p));
        for (int idx = threadIdx.x; idx < KT * DH; idx += blockDim.x) {
            const int jj = idx / DH, e = idx - jj * DH;
            const bool ok = jj < jn && e < d_h;
            ks[jj][e] = ok ? to_f32(kp[(size_t)(j0 + jj) * d_h + e]) : 0.f;
            vs[jj][e] = ok ? to_f32(vp[(size_t)(j0 + jj) * d_h + e]) : 0.f;
        }
        __syncthreads();
        if (live) {
            for (int jj = 0; jj < jn; ++jj) {
                if (!km[jj] || (causal && j0 + jj > r)) continue;  // masked key
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
    const float inv = den > 0.f ? w / den : 0.f;  // a row with no admissible key contributes nothing
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

// ---------------------------------------------------------------------------------------------
// MFMA attention (bf16, d_h in {32, 64, 128}), Eq. 33-34.  One wave owns 32 query rows of one unit and
// walks key tiles of 64, online softmax in fp32 (base 2: q arrives pre-scaled by log2(e)/sqrt(d_h)).
//
// Layout.  The scores are computed TRANSPOSED, S^T = K Q^T (v_mfma_f32_32x32x16_bf16), so that an
// accumulator lane holds one query column: the row max / row sum of the softmax are in-lane
// reductions plus one exchange with the partner lane (lane ^ 32), and the probabilities, converted
// in place, already ARE the B operand of the second product O^T = V^T P^T (the k-slots of an MFMA
// operand may hold any permutation of K as long as both operands agree, so V^T is read with the
// accumulator's key order: keys 16s+4h..+4 and 16s+8+4h..+4 for k-step s, half-wave h).
//
// What the kernel is bound by is the vector ALU work of the softmax, not the matrix pipe, so that work
// is kept to a max, an exp2, an add and half a convert per score:
//  * P V runs in fp16 (v_mfma_f32_32x32x16_f16): probabilities carry 11 significant bits, enough for
//    the 2e-2 bound with one MFMA pass (a bf16 P needs a (hi, lo) pair: twice the MFMAs plus the split
//    arithmetic).  The projection kernel writes V as fp16 straight from its fp32 accumulators (VF16;
//    11 significant bits instead of bf16's 8, |v| up to 65504).  When the caller needs V in bf16 (the
//    backward pass) the kernel converts bf16 -> fp16 while it stages the tile instead (exact for
//    |v| in [6.1e-5, 65504]).
//  * The running maximum is subtracted by the matrix pipe: the score accumulators are initialised
//    with -m instead of 0.  As long as no score of a tile exceeds the running maximum by more than
//    2^8 the tile needs no rescaling at all (p = exp2(s - m) <= 256 fits fp16 and fp32 sums); only
//    when one does (always on the first tile) the maximum moves and O and the row sum are rescaled.
//  * KSPLIT waves share a query block and take key tiles KSPLIT apart, so that a compute unit holds
//    two waves per SIMD also when the grid has only one wave of queries per SIMD: one wave's softmax
//    then runs under another's MFMAs.  Their (max, sum, O) triples are merged through LDS at the end.
// K and V tiles [key][d_h] are staged through double-buffered LDS as 16-byte row copies; the V^T
// fragments come out of the [key][d_h] tile through the transposing LDS read.
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));

__device__ __forceinline__ uint32_t pack2_f16(float a, float b)
{
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(a, b));  // toward zero: never rounds up to inf
}

// One key tile of 64 keys for the 32 queries of a wave: scores, masks, the lazy running maximum, probabilities and
// O^T += V^T P^T.  kfrag(t, ks) gives the K fragment of accumulator tile t (keys t*32 + lane%32) for k-step ks,
// vfrag(s4, td) the V^T fragment of key step s4 for head-dim block td; km points at the tile's padding flags
// (one byte per key) or is NULL.  The staging of K and V is the caller's.
template <int DH, typename KF, typename VF>
__device__ __forceinline__ void attention_tile(const bf16x8_t (&qf)[DH / 16], f32x16_t (&oacc)[DH / 32], float &mrun, float &lsum, int kt,
                                               int l_a, int qrow, int qrow_first, bool causal, const unsigned char *km, int lane,
                                               KF kfrag, VF vfrag)
{
    constexpr int BKV = 64;
    constexpr float TAU = 8.0f;
    const int lh = lane >> 5;
    const bool masked = km != nullptr;
    // S^T tile: [64 keys x 32 queries] as two 32x32 accumulators, started at -m
    const float moff = mrun == -INFINITY ? 0.f : mrun;
    f32x16_t sacc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int q = 0; q < 16; ++q) sacc[t][q] = -moff;
#pragma unroll
    for (int ks = 0; ks < DH / 16; ++ks)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const bf16x8_t kf = kfrag(t, ks);
            sacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], sacc[t], 0, 0, 0);
        }
    // accumulator register q of tile t is key kt*64 + t*32 + (q/4)*8 + lh*4 + q%4.  Masks: a wave-uniform
    // test whether the tile can hold an inadmissible key for any query of the wave, then straight-line
    // selects (accumulators must not cross divergent branches).
    if ((kt + 1) * BKV > l_a || masked || (causal && (kt + 1) * BKV > qrow_first + 1)) {
        uint32_t kmw[2][4];   // the padding flags of this lane's keys, four consecutive keys per word
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq)
                kmw[t][gq] = masked ? *reinterpret_cast<const uint32_t *>(km + t * 32 + gq * 8 + lh * 4) : 0x01010101u;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int key = kt * BKV + t * 32 + (q >> 2) * 8 + lh * 4 + (q & 3);
                const bool ok = key < l_a && (!causal || key <= qrow) && ((kmw[t][q >> 2] >> ((q & 3) * 8)) & 0xFFu) != 0;
                sacc[t][q] = ok ? sacc[t][q] : -INFINITY;
            }
    }
    float tmax = -INFINITY;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int q = 0; q < 16; ++q) tmax = fmaxf(tmax, sacc[t][q]);
    {   // largest score of the tile, relative to the running maximum: the other half-wave's value through
        // v_permlane32_swap (lanes 32-63 of the first result and lanes 0-31 of the second hold the partner's)
        const uint32_t tb = __float_as_uint(tmax);
        const auto sw = __builtin_amdgcn_permlane32_swap(tb, tb, false, false);
        tmax = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
    }
    // the maximum moves only when a score exceeds it by more than 2^TAU, or when there is none yet
    const bool move = tmax > TAU || (mrun == -INFINITY && tmax > -INFINITY);
    if (__builtin_amdgcn_ballot_w64(move) != 0) {   // wave-uniform: rare after the first tile
        if (move) {
            const float corr = mrun == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(-tmax);
            mrun = moff + tmax;
            lsum *= corr;
#pragma unroll
            for (int t = 0; t < DH / 32; ++t)
#pragma unroll
                for (int q = 0; q < 16; ++q) oacc[t][q] *= corr;
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int q = 0; q < 16; ++q) sacc[t][q] -= tmax;
        }
    }
    float psum = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const float pv = __builtin_amdgcn_exp2f(sacc[t][q]);   // exp2(-inf) = 0 for masked keys
            sacc[t][q] = pv;
            psum += pv;
        }
    lsum += psum;

    // O^T += V^T P^T over the 64 keys of the tile: four k-steps of 16 keys
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
        const int t = s4 >> 1, r0 = (s4 & 1) * 8;
        uint32_t ph[4];  // two probabilities per word, fp16
#pragma unroll
        for (int e = 0; e < 4; ++e) ph[e] = pack2_f16(sacc[t][r0 + 2 * e], sacc[t][r0 + 2 * e + 1]);
        const f16x8_t pf = __builtin_bit_cast(f16x8_t, make_uint4(ph[0], ph[1], ph[2], ph[3]));
#pragma unroll
        for (int td = 0; td < DH / 32; ++td) {
            const f16x8_t vf = vfrag(s4, td);
            oacc[td] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf, oacc[td], 0, 0, 0);
        }
    }
}

// End of an attention workgroup: the key splits are merged (splits 1.. park their (max, row sum, O^T) in LDS, whose
// tile buffers are free once the key loop has ended on a barrier; split 0 folds them in, in split order), then
// split 0 normalises, applies the row's gate weight and writes o as a (hi, lo) bf16 pair and, if asked, the
// base-2 log-sum-exp of the row.
template <int DH, int NQ, int KSPLIT>
__device__ __forceinline__ void attention_finish(const SmhaArgs &a, unsigned char *lds_raw, int split, int qg, int lane, int g, int qrow,
                                                 int l_a, float w, f32x16_t (&oacc)[DH / 32], float mrun, float lsum)
{
    const int lh = lane >> 5;
    if constexpr (KSPLIT > 1) {
        float *mg = reinterpret_cast<float *>(lds_raw);
        constexpr int SLOT = DH / 2 + 2;   // floats per lane
        if (split > 0) {
            float *dst = mg + ((size_t)((split - 1) * NQ + qg) * 64 + lane) * SLOT;
            dst[0] = mrun;
            dst[1] = lsum;
#pragma unroll
            for (int t = 0; t < DH / 32; ++t)
#pragma unroll
                for (int q = 0; q < 16; ++q) dst[2 + t * 16 + q] = oacc[t][q];
        }
        __syncthreads();
        if (split > 0) return;
#pragma unroll
        for (int s = 1; s < KSPLIT; ++s) {
            const float *src = mg + ((size_t)((s - 1) * NQ + qg) * 64 + lane) * SLOT;
            const float m1 = src[0], l1 = src[1];
            const float mf = fmaxf(mrun, m1);
            // a side that has seen no admissible key (max = -inf) contributes nothing
            const float c0 = mrun == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mrun - mf);
            const float c1 = m1 == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m1 - mf);
            lsum = lsum * c0 + l1 * c1;
#pragma unroll
            for (int t = 0; t < DH / 32; ++t)
#pragma unroll
                for (int q = 0; q < 16; ++q) oacc[t][q] = oacc[t][q] * c0 + src[2 + t * 16 + q] * c1;
            mrun = mf;
        }
    }

    if (qrow >= l_a) return;
    lsum += __shfl_xor(lsum, 32, 64);
    const float inv = lsum > 0.f ? w / lsum : 0.f;  // a row with no admissible key contributes nothing
    if (a.lse && lh == 0) a.lse[(size_t)g * l_a + qrow] = lsum > 0.f ? mrun + log2f(lsum) : 0.f;
    bf16_t *o = static_cast<bf16_t *>(a.o) + ((size_t)g * l_a + qrow) * DH;
    bf16_t *o_lo = static_cast<bf16_t *>(a.o_lo) + ((size_t)g * l_a + qrow) * DH;
    // accumulator register q of tile td is head-dim index td*32 + (q/4)*8 + lh*4 + q%4.
    // o is written as hi = bf16(o) and lo = bf16(o - hi): the out-projection contracts both.
#pragma unroll
    for (int td = 0; td < DH / 32; ++td)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            uint32_t hi[2], lo[2];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const float v0 = oacc[td][i4 * 4 + 2 * e] * inv, v1 = oacc[td][i4 * 4 + 2 * e + 1] * inv;
                hi[e] = pack2_bf16(v0, v1);
                lo[e] = pack2_bf16(v0 - __uint_as_float(hi[e] << 16), v1 - __uint_as_float(hi[e] & 0xFFFF0000u));
            }
            *reinterpret_cast<uint2 *>(o + td * 32 + i4 * 8 + lh * 4) = make_uint2(hi[0], hi[1]);
            *reinterpret_cast<uint2 *>(o_lo + td * 32 + i4 * 8 + lh * 4) = make_uint2(lo[0], lo[1]);
        }
}

template <int DH, int NQ, int KSPLIT, bool VF16>
__global__ __launch_bounds__(NQ *KSPLIT * 64) void attention_mfma_kernel(SmhaArgs a)
{
    constexpr int BKV = 64, KP = DH + 8, VP = 2 * b_pitch_dwords(DH), NTH = NQ * 64;  // NTH: threads that stage one split's tiles
    constexpr int CHUNKS = BKV * DH / 8, PER_T = (CHUNKS + NTH - 1) / NTH;
    constexpr int PD = 3;   // register sets of the K/V prefetch
    constexpr int K_BYTES = 2 * BKV * KP * 2, V_BYTES = 2 * BKV * VP * 2, SPLIT_BYTES = K_BYTES + V_BYTES + 2 * BKV;
    constexpr int MERGE_BYTES = (KSPLIT - 1) * NQ * 64 * (DH / 2 + 2) * 4;
    constexpr int LDS_BYTES = KSPLIT * SPLIT_BYTES > MERGE_BYTES ? KSPLIT * SPLIT_BYTES : MERGE_BYTES;
    __shared__ __align__(16) unsigned char lds_raw[LDS_BYTES];

    const int l_p = a.l / a.m, l_a = a.c * l_p;
    // Workgroup -> (unit, query block).  Hardware deals consecutive workgroup ids round-robin over the 8
    // XCDs, each with its own L2: the query blocks of one unit are given ids 8 apart, so that a unit's K and
    // V are fetched into one L2 only (units in groups of 8; a ragged last group keeps the plain order).
    int g, qblk;
    {
        const int nqb = (l_a + 32 * NQ - 1) / (32 * NQ), units = a.b * a.k, id = blockIdx.x;
        const int full = (units / 8) * 8 * nqb;   // ids that belong to whole groups of 8 units
        if (id < full) {
            const int grp = id / (8 * nqb), rem = id - grp * 8 * nqb;
            g = grp * 8 + (rem & 7);
            qblk = rem >> 3;
        } else {
            const int rem = id - full;
            g = (units / 8) * 8 + rem / nqb;
            qblk = rem % nqb;
        }
    }
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: tile tests stay scalar
    const int split = wave / NQ, qg = wave - split * NQ, stid = tid - split * NTH;  // key split, query group, thread within the split
    const int lr = lane & 31, lh = lane >> 5;
    const int qrow = qblk * (32 * NQ) + qg * 32 + lr;
    unsigned char *sbase = lds_raw + (size_t)split * SPLIT_BYTES;
    uint16_t(*Ks)[BKV][KP] = reinterpret_cast<uint16_t(*)[BKV][KP]>(sbase);
    uint16_t(*Vs)[BKV][VP] = reinterpret_cast<uint16_t(*)[BKV][VP]>(sbase + K_BYTES);   // fp16, [key][d_h]
    unsigned char(*Km)[BKV] = reinterpret_cast<unsigned char(*)[BKV]>(sbase + K_BYTES + V_BYTES);
    const bf16_t *Q = static_cast<const bf16_t *>(a.q) + (size_t)g * l_a * DH;
    const bf16_t *Kg = static_cast<const bf16_t *>(a.kk) + (size_t)g * l_a * DH;
    const bf16_t *Vg = static_cast<const bf16_t *>(a.v) + (size_t)g * l_a * DH;

    // gate weight of this row (Eq. 36 with the optional gate flags): two dependent lookups, started
    // here so that they complete under the key loop instead of in front of the output stores
    float w = 1.0f;
    if (split == 0) {
        const int bb = g / a.k, i = clampi(a.expert_idx[g], a.n);
        if ((a.flags & F_GATE_EXPERT) && a.expert_gate) w *= a.expert_gate[(size_t)bb * a.n + i];
        if ((a.flags & F_GATE_PATCH) && a.patch_gate) {
            const int p = clampi(a.patch_idx[((size_t)bb * a.n + i) * a.c + min(qrow, l_a - 1) / l_p], a.m);
            w *= a.patch_gate[((size_t)bb * a.n + i) * a.m + p];
        }
    }

    bf16x8_t qf[DH / 16];
#pragma unroll
    for (int ks = 0; ks < DH / 16; ++ks) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (qrow < l_a) v = *reinterpret_cast<const uint4 *>(Q + (size_t)qrow * DH + ks * 16 + lh * 8);
        qf[ks] = __builtin_bit_cast(bf16x8_t, v);
    }

    f32x16_t oacc[DH / 32];
#pragma unroll
    for (int t = 0; t < DH / 32; ++t)
#pragma unroll
        for (int q = 0; q < 16; ++q) oacc[t][q] = 0.f;
    float mrun = -INFINITY, lsum = 0.f;   // running maximum of this query (both half-waves agree), this lane's part of the row sum

    const bool causal = (a.flags & F_CAUSAL) != 0, masked = a.pad_mask != nullptr;
    const int nkt_all = (l_a + BKV - 1) / BKV;
    // K/V tiles travel global -> registers -> LDS.  A tile's loads are issued PD - 1 iterations before the
    // tile is used (PD register sets): one iteration of a key split is shorter than a memory round trip.
    struct Staged {   // plain words, moved one by one: whole-vector copies of a local array would be a memcpy, which
        uint32_t k[PER_T][4], v[PER_T][4];   // keeps the array out of the register file
        unsigned char km;
    };
    Staged set0, set1, set2;   // separate objects: each one small enough to live in registers
    // Loads are issued for every iteration, also past the last tile (the last tile again, never stored),
    // with clamped addresses instead of guards: straight-line code whose outstanding loads the
    // compiler can count, so a wait for one tile leaves the younger tiles in flight.
    static_assert(CHUNKS % NTH == 0, "every staging thread moves the same number of pieces");
    // Element offset of piece i in tile t: ((t * BKV + row_i) * DH + kc_i * 8), clamped to the same piece of
    // the last key (keys past l_a repeat the last key: their scores are masked to -inf below, so they get
    // probability 0 against finite V rows; zeroing the registers instead would make every load wait).
    uint32_t piece[PER_T], piece_last[PER_T];
#pragma unroll
    for (int i = 0; i < PER_T; ++i) {
        const int c = stid + i * NTH;
        piece[i] = (uint32_t)(c / (DH / 8)) * DH + (c % (DH / 8)) * 8;
        piece_last[i] = (uint32_t)(l_a - 1) * DH + (c % (DH / 8)) * 8;
    }
    auto load_global = [&](Staged &sr, int tile) {
        if (masked && stid < BKV) {
            const int key = tile * BKV + stid;
            sr.km = key < l_a && key_is_token(a, g, min(key, l_a - 1), l_p);
        }
        const uint32_t t0 = (uint32_t)min(tile, nkt_all) * (BKV * DH);   // a tile past the end: clamped below, never stored
#pragma unroll
        for (int i = 0; i < PER_T; ++i) {
            const uint32_t at = min(t0 + piece[i], piece_last[i]);
            const uint4 kq = *reinterpret_cast<const uint4 *>(Kg + at), vq = *reinterpret_cast<const uint4 *>(Vg + at);
            sr.k[i][0] = kq.x; sr.k[i][1] = kq.y; sr.k[i][2] = kq.z; sr.k[i][3] = kq.w;
            sr.v[i][0] = vq.x; sr.v[i][1] = vq.y; sr.v[i][2] = vq.z; sr.v[i][3] = vq.w;
        }
    };
    auto store_lds = [&](const Staged &sr, int buf) {
        if (masked && stid < BKV) Km[buf][stid] = sr.km;
#pragma unroll
        for (int i = 0; i < PER_T; ++i) {
            const int c = stid + i * NTH;
            {
                *reinterpret_cast<uint4 *>(&Ks[buf][c / (DH / 8)][(c % (DH / 8)) * 8]) = make_uint4(sr.k[i][0], sr.k[i][1], sr.k[i][2], sr.k[i][3]);
                const uint32_t u[4] = {sr.v[i][0], sr.v[i][1], sr.v[i][2], sr.v[i][3]};
                uint32_t h[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    // a bf16 v: widen to fp32 (a shift), then narrow; exact whenever fp16 can hold the value
                    if constexpr (VF16) h[e] = u[e];
                    else h[e] = pack2_f16(__uint_as_float(u[e] << 16), __uint_as_float(u[e] & 0xFFFF0000u));
                }
                *reinterpret_cast<uint4 *>(&Vs[buf][c / (DH / 8)][(c % (DH / 8)) * 8]) = make_uint4(h[0], h[1], h[2], h[3]);
            }
        }
    };

    // under the causal mask no query of this workgroup sees keys past the workgroup's last row
    const int key_end = causal ? min(l_a, (qblk + 1) * 32 * NQ) : l_a;
    const int nkt = (key_end + BKV - 1) / BKV;
    const int nit = (nkt + KSPLIT - 1) / KSPLIT;   // iterations: split s takes tiles s, s + KSPLIT, ...
    auto tile_of = [&](int it) { return it * KSPLIT + split; };   // this split's it-th tile (exists if < nkt)
    set0.km = set1.km = set2.km = 1;
    load_global(set0, tile_of(0));
    load_global(set1, tile_of(1));
    store_lds(set0, 0);
    __syncthreads();
    // one iteration; J = it % PD picks the register sets at compile time (arrays indexed by a run-time
    // value would leave the register file)
    auto iteration = [&](auto jc, int it) {
        constexpr int J = decltype(jc)::value;
        const int kt = tile_of(it), buf = it & 1;
        Staged &fill = J == 0 ? set2 : (J == 1 ? set0 : set1), &drain = J == 0 ? set1 : (J == 1 ? set2 : set0);
        load_global(fill, tile_of(it + PD - 1));
        if (kt < nkt) {
            attention_tile<DH>(qf, oacc, mrun, lsum, kt, l_a, qrow, qblk * (32 * NQ) + qg * 32, causal, masked ? &Km[buf][0] : nullptr, lane,
                               [&](int t, int ks) { return *reinterpret_cast<const bf16x8_t *>(&Ks[buf][t * 32 + lr][ks * 16 + lh * 8]); },
                               [&](int s4, int td) {
                                   // V^T fragment for head-dim column td*32 + lr: keys 16*s4 + 4*lh + 0..3, then + 8
                                   const uint16_t *vsrc = &Vs[buf][s4 * 16 + lh * 4 + ((lane & 15) >> 2)][td * 32 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4];
                                   const uint2 v0 = lds_read_tr4(vsrc);
                                   const uint2 v1 = lds_read_tr4(vsrc + 8 * VP);
                                   return __builtin_bit_cast(f16x8_t, make_uint4(v0.x, v0.y, v1.x, v1.y));
                               });
        }
        if (tile_of(it + 1) < nkt) store_lds(drain, buf ^ 1);
        __syncthreads();
    };
    static_assert(PD == 3, "the loop below names the register sets");
    for (int it0 = 0; it0 < nit; it0 += PD) {   // nit is uniform over the workgroup
        iteration(std::integral_constant<int, 0>{}, it0);
        if (it0 + 1 < nit) iteration(std::integral_constant<int, 1>{}, it0 + 1);
        if (it0 + 2 < nit) iteration(std::integral_constant<int, 2>{}, it0 + 2);
    }

    attention_finish<DH, NQ, KSPLIT>(a, lds_raw, split, qg, lane, g, qrow, l_a, w, oacc, mrun, lsum);
}

// The same kernel with K and V tiles copied from global memory straight into LDS (global_load_lds_dwordx4:
// 16 bytes per lane, the 64 lanes of an instruction fill 1 KiB of consecutive LDS), three tiles deep: no
// staging registers, no LDS store instructions and no converts in the loop, and a wave waits for a tile only
// when it needs it.  What that takes: V already in fp16 in memory (the projection kernel writes it so), no
// padding mask (its per-key lookups are ordinary loads, whose compiler-placed waits would drain the copies in
// flight: masked calls take the register-staged kernel), and unpadded tiles, so bank conflicts are avoided
// by permuting which 16-byte piece of a row an LDS slot receives (every lane supplies its own global
// address): K slot (r, pos) <- piece pos ^ ((r / (16/CK)) % CK), the rule for tiles read as row fragments; V
// slot (r, pos) <- piece pos ^ ((r & 3) << 2) for 256-byte rows (d_h = 128) and pos ^ (((r >> 1) & 1) << 2) for
// 128-byte rows (d_h = 64), the rule for tiles read with the transposing LDS read.  The copies are inline
// assembly that the compiler cannot count, so their completion is waited for by hand (they complete in
// issue order): at the top of an iteration at most the copies of the STAGES-2 younger tiles may be
// outstanding, then one barrier publishes every wave's part of the tile and frees the buffer of the tile
// before for the copies issued right after it.
template <int DH, int NQ, int KSPLIT>
__global__ __launch_bounds__(NQ *KSPLIT * 64) void attention_dma_kernel(SmhaArgs a)
{
    static_assert(DH == 64 || DH == 128, "piece permutations are written for 128- and 256-byte rows");
    constexpr int BKV = 64, STAGES = 4;
    constexpr int CK = DH / 8;                        // 16-byte pieces per row
    constexpr int RPI = 64 / CK;                      // rows one copy instruction covers
    constexpr int TILE_BYTES = BKV * DH * 2, INSTR = TILE_BYTES / 1024;
    constexpr int PER_W = INSTR / NQ;                 // copy instructions per wave, tile and operand
    static_assert(INSTR % NQ == 0, "every wave of a split issues the same number of copies");
    constexpr int SPLIT_BYTES = STAGES * 2 * TILE_BYTES;
    constexpr int MERGE_BYTES = (KSPLIT - 1) * NQ * 64 * (DH / 2 + 2) * 4;
    constexpr int LDS_BYTES = KSPLIT * SPLIT_BYTES > MERGE_BYTES ? KSPLIT * SPLIT_BYTES : MERGE_BYTES;
    __shared__ __align__(1024) unsigned char lds_raw[LDS_BYTES];

    const int l_p = a.l / a.m, l_a = a.c * l_p;
    int g, qblk;   // workgroup -> (unit, query block): the query blocks of a unit share an XCD (see attention_mfma_kernel)
    {
        const int nqb = (l_a + 32 * NQ - 1) / (32 * NQ), units = a.b * a.k, id = blockIdx.x;
        const int full = (units / 8) * 8 * nqb;
        if (id < full) {
            const int grp = id / (8 * nqb), rem = id - grp * 8 * nqb;
            g = grp * 8 + (rem & 7);
            qblk = rem >> 3;
        } else {
            const int rem = id - full;
            g = (units / 8) * 8 + rem / nqb;
            qblk = rem % nqb;
        }
    }
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int split = wave / NQ, qg = wave - split * NQ;
    const int lr = lane & 31, lh = lane >> 5;
    const int qrow = qblk * (32 * NQ) + qg * 32 + lr;
    unsigned char *sbase = lds_raw + (size_t)split * SPLIT_BYTES;   // stage s: K tile at s * 2 * TILE_BYTES, V tile after it
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)sbase;
    const bf16_t *Q = static_cast<const bf16_t *>(a.q) + (size_t)g * l_a * DH;
    const uint16_t *Kg = static_cast<const uint16_t *>(a.kk) + (size_t)g * l_a * DH;
    const uint16_t *Vg = static_cast<const uint16_t *>(a.v) + (size_t)g * l_a * DH;

    float w = 1.0f;   // gate weight of this row (Eq. 36), looked up early
    if (split == 0) {
        const int bb = g / a.k, i = clampi(a.expert_idx[g], a.n);
        if ((a.flags & F_GATE_EXPERT) && a.expert_gate) w *= a.expert_gate[(size_t)bb * a.n + i];
        if ((a.flags & F_GATE_PATCH) && a.patch_gate) {
            const int p = clampi(a.patch_idx[((size_t)bb * a.n + i) * a.c + min(qrow, l_a - 1) / l_p], a.m);
            w *= a.patch_gate[((size_t)bb * a.n + i) * a.m + p];
        }
    }
    bf16x8_t qf[DH / 16];
#pragma unroll
    for (int ks = 0; ks < DH / 16; ++ks) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (qrow < l_a) v = *reinterpret_cast<const uint4 *>(Q + (size_t)qrow * DH + ks * 16 + lh * 8);
        qf[ks] = __builtin_bit_cast(bf16x8_t, v);
    }
    f32x16_t oacc[DH / 32];
#pragma unroll
    for (int t = 0; t < DH / 32; ++t)
#pragma unroll
        for (int q = 0; q < 16; ++q) oacc[t][q] = 0.f;
    float mrun = -INFINITY, lsum = 0.f;

    auto v_swz = [](int r) { return (DH == 128 ? (r & 3) : ((r >> 1) & 1)) << 2; };
    // Copy roles.  Instruction j of this wave fills 1 KiB block qg * PER_W + j of a tile: lane -> slot (row, pos).
    // Element offsets inside the unit's K (V) array, for tile 0; a tile adds BKV * DH.  Keys past l_a repeat
    // the last key (their scores are masked, so they get probability 0 against finite V rows).
    uint32_t k_off[PER_W], v_off[PER_W], k_last[PER_W], v_last[PER_W];
#pragma unroll
    for (int j = 0; j < PER_W; ++j) {
        const int r = (qg * PER_W + j) * RPI + lane / CK, pos = lane % CK;
        const int kp = pos ^ ((r / (16 / CK)) % CK), vp = pos ^ v_swz(r);
        k_off[j] = (uint32_t)r * DH + kp * 8;
        v_off[j] = (uint32_t)r * DH + vp * 8;
        k_last[j] = (uint32_t)(l_a - 1) * DH + kp * 8;
        v_last[j] = (uint32_t)(l_a - 1) * DH + vp * 8;
    }
    const bool causal = (a.flags & F_CAUSAL) != 0;
    const int nkt_all = (l_a + BKV - 1) / BKV;
    const int key_end = causal ? min(l_a, (qblk + 1) * 32 * NQ) : l_a;   // no query of this workgroup sees later keys
    const int nkt = (key_end + BKV - 1) / BKV;
    const int nit = (nkt + KSPLIT - 1) / KSPLIT;   // iterations: split s takes tiles s, s + KSPLIT, ...
    auto tile_of = [&](int it) { return it * KSPLIT + split; };
    // copies are issued for every iteration, also past the last tile (clamped to the end, never read): the
    // number outstanding is then the same in every iteration
    auto issue = [&](int it, int stage) {
        const uint32_t t0 = (uint32_t)min(tile_of(it), nkt_all) * (BKV * DH);
        const uint32_t dst = lds_base + stage * (2 * TILE_BYTES) + qg * PER_W * 1024;
#pragma unroll
        for (int j = 0; j < PER_W; ++j) {
            dma_load16(Kg + min(t0 + k_off[j], k_last[j]), dst + j * 1024);
            dma_load16(Vg + min(t0 + v_off[j], v_last[j]), dst + TILE_BYTES + j * 1024);
        }
    };
#pragma unroll
    for (int q = 0; q < STAGES - 1; ++q) issue(q, q);
    // fragment offsets (bytes inside a stage): K row fragments, V^T through the transposing read
    const int vx = (lane & 15) >> 2;   // row of the 4-row group this lane points at
    int stage = 0, fill = STAGES - 1;
    for (int it = 0; it < nit; ++it) {   // nit is uniform over the workgroup
        dma_wait<(STAGES - 2) * 2 * PER_W>();
        __syncthreads();
        issue(it + STAGES - 1, fill);
        const int kt = tile_of(it);
        if (kt < nkt) {
            const unsigned char *kb = sbase + stage * (2 * TILE_BYTES), *vb = kb + TILE_BYTES;
            attention_tile<DH>(qf, oacc, mrun, lsum, kt, l_a, qrow, qblk * (32 * NQ) + qg * 32, causal, nullptr, lane,
                               [&](int t, int ks) {
                                   const int r = t * 32 + lr;
                                   return *reinterpret_cast<const bf16x8_t *>(kb + r * (DH * 2) + (((ks * 2 + lh) ^ ((r / (16 / CK)) % CK)) * 16));
                               },
                               [&](int s4, int td) {
                                   // keys 16*s4 + 4*lh + vx, then + 8 (the same permutation of both rows), head-dim columns
                                   // td*32 + ((lane>>4)&1)*16 + (lane&3)*4 .. +3
                                   const int r = s4 * 16 + lh * 4 + vx;
                                   const int piece = (td * 4 + ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1)) ^ v_swz(r);
                                   const uint16_t *vsrc = reinterpret_cast<const uint16_t *>(vb + r * (DH * 2) + piece * 16 + (lane & 1) * 8);
                                   const uint2 v0 = lds_read_tr4(vsrc);
                                   const uint2 v1 = lds_read_tr4(vsrc + 8 * DH);
                                   return __builtin_bit_cast(f16x8_t, make_uint4(v0.x, v0.y, v1.x, v1.y));
                               });
        }
        stage = stage + 1 == STAGES ? 0 : stage + 1;
        fill = fill + 1 == STAGES ? 0 : fill + 1;
    }
    dma_wait<0>();     // the copies past the last tile
    __syncthreads();   // every wave is done with the tiles: LDS is free for the merge
    attention_finish<DH, NQ, KSPLIT>(a, lds_raw, split, qg, lane, g, qrow, l_a, w, oacc, mrun, lsum);
}

// Launch shape: NQ waves of 32 queries per workgroup (more share K/V tiles, fewer give more workgroups:
// at least one workgroup per compute unit if possible), KSPLIT key splits so that the grid holds two
// waves per SIMD (2048 waves) where the key tiles allow it.
template <int DH, int NQ, int KSPLIT> static void launch_attention_shape(const SmhaArgs &a, hipStream_t st)
{
    const int l_a = a.c * (a.l / a.m), units = a.b * a.k;
    const dim3 grid(((l_a + 32 * NQ - 1) / (32 * NQ)) * units), block(NQ * KSPLIT * 64);
    if (a.keep_v_bf16) {
        hipLaunchKernelGGL((attention_mfma_kernel<DH, NQ, KSPLIT, false>), grid, block, 0, st, a);
        return;
    }
    // (LDS: stages x (K + V tile) per split; every wave the same number of copies; the wait count fits its field)
    if constexpr ((DH == 64 || DH == 128) && KSPLIT * 4 * 2 * 64 * DH * 2 <= 160 * 1024 && (64 * DH * 2 / 1024) % NQ == 0 &&
                  2 * 2 * (64 * DH * 2 / 1024 / NQ) <= 63) {
        if (!a.pad_mask) {   // V in fp16, no padding mask: tiles copied straight into LDS
            hipLaunchKernelGGL((attention_dma_kernel<DH, NQ, KSPLIT>), grid, block, 0, st, a);
            return;
        }
    }
    hipLaunchKernelGGL((attention_mfma_kernel<DH, NQ, KSPLIT, true>), grid, block, 0, st, a);
}

template <int DH> static hipError_t launch_attention_mfma_dh(const SmhaArgs &a, hipStream_t st)
{
    const int l_a = a.c * (a.l / a.m), units = a.b * a.k;
    const long waves = (long)units * ((l_a + 31) / 32);
    const int nkt = (l_a + 63) / 64;
    int ks = 1;
    while (ks < 4 && waves * ks < 2048 && 2 * ks <= nkt) ks *= 2;
    if (DH > 32 && ks > 2) ks = 2;     // LDS: four splits fit a compute unit only with d_h = 32 tiles
    int nq = 4;
    while (nq > 1 && ((l_a + 32 * nq - 1) / (32 * nq)) * (long)units < 256) nq >>= 1;
    if (nq == 4 && ks == 4) ks = 2;    // at most 8 waves per workgroup
#define UOE_ATT(NQ, KS) launch_attention_shape<DH, NQ, KS>(a, st)
    if (nq == 4) { if (ks == 1) UOE_ATT(4, 1); else UOE_ATT(4, 2); }
    else if (nq == 2) {
        if (ks == 1) UOE_ATT(2, 1);
        else if (ks == 2) UOE_ATT(2, 2);
        else if constexpr (DH == 32) UOE_ATT(2, 4);
    } else {
        if (ks == 1) UOE_ATT(1, 1);
        else if (ks == 2) UOE_ATT(1, 2);
        else if constexpr (DH == 32) UOE_ATT(1, 4);
    }
#undef UOE_ATT
    return hipGetLastError();
}

static hipError_t launch_attention_mfma(const SmhaArgs &a, hipStream_t st)
{
    if (a.d_h == 32) return launch_attention_mfma_dh<32>(a, st);
    if (a.d_h == 64) return launch_attention_mfma_dh<64>(a, st);
    return launch_attention_mfma_dh<128>(a, st);
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
    qp.q_scale = 1.0f;
    qp.nout = 3;
    qp.q32 = nullptr;
    return qp;
}

template <typename T> static OutProjProblem<T> make_outproj(const SmhaArgs &a)
{
    OutProjProblem<T> op;
    op.o = static_cast<const T *>(a.o);
    op.o_lo = nullptr;
    op.parts = 1;
    op.wo = static_cast<const T *>(a.wo);
    op.x = static_cast<const T *>(a.x);
    op.expert_idx = a.expert_idx;
    op.patch_idx = a.patch_idx;
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
    if (!(a.skip & SMHA_STEP_QKV)) {
        if ((err = launch_gemm_generic<T>(make_qkv<T>(a), units, l_a, 3 * a.d_h, st)) != hipSuccess) return err;
        if ((err = launch_rope<T>(a, st)) != hipSuccess) return err;
    }
    if (!(a.skip & SMHA_STEP_ATTENTION) && (err = launch_attention_generic<T>(a, st)) != hipSuccess) return err;
    if (a.skip & SMHA_STEP_OUT) return hipSuccess;
    if ((err = launch_inverse_map(a, st)) != hipSuccess) return err;
    return launch_gemm_generic<T>(make_outproj<T>(a), a.b * a.m, l_p, a.d, st);
}

// Tile choice of the pipelined output-stationary contraction (out-projection of SMHA, second layer
// of the data-selected UoME).  A (sample, patch) group is a short chain of dependent steps (find the
// experts that picked the patch, fetch their rows, a few K-steps, add the residual), so with many
// short groups what counts is how many of them a CU holds at once: two-wave workgroups with two
// stage buffers (five per CU) beat four-wave ones on the ViT shape (out-projection 30 -> 22 us; one
// workgroup over the whole row width, one-wave workgroups and 64-column tiles were all slower),
// while the LM shape's 128 groups are better off with four waves and every K-step in flight.
template <typename OP> static hipError_t launch_outproj_dma(const OP &op, int groups, int l_p, int d, hipStream_t st)
{
    if (groups >= 512 && l_p <= 32) return launch_gemm_dma<OP, 32, 128, 32, 1, 2, 2, 4>(op, groups, l_p, d, st);
    if (l_p <= 32) return launch_gemm_dma<OP, 32, 128, 32, 1, 4, 4, 2>(op, groups, l_p, d, st);
    // many 64-row groups: four workgroups per CU with two stage buffers each (more of the short dependent
    // chains in flight: out-projection of the large shape 40.5 -> 35.9 us)
    if ((long)groups * ((d + 127) / 128) >= 2048) return launch_gemm_dma<OP, 64, 128, 32, 2, 2, 2, 4>(op, groups, l_p, d, st);
    return launch_gemm_dma<OP, 64, 128, 32, 2, 2, 4, 2>(op, groups, l_p, d, st);
}

// projections, rotary embedding and attention of the MFMA path
static hipError_t smha_mfma_qkv_attention(const SmhaArgs &a, hipStream_t st)
{
    typedef QkvProblem<bf16_t> QP;
    const int l_p = a.l / a.m, l_a = a.c * l_p, units = a.b * a.k;
    hipError_t err;
    QP qp = make_qkv<bf16_t>(a);
    // the MFMA kernel addresses one unit's keys with 32-bit element offsets
    const bool mfma_attn = (a.d_h == 32 || a.d_h == 64 || a.d_h == 128) && (long)l_a * a.d_h < (1L << 31);
    if (mfma_attn) qp.q_scale = 1.4426950408889634f / sqrtf((float)a.d_h);  // base-2 softmax in the MFMA kernel
    qp.v_f16 = mfma_attn && !a.keep_v_bf16;
    // one workgroup row-tile computes q, k and v together so the gathered rows are read once
    // 128-row tiles for long units (measured faster from l_a = 512 up), 32-row tiles for short ones
    auto projections = [&]() -> hipError_t {
    const bool tall = l_a >= 256 && (long)units * ((l_a + 127) / 128) >= 128, k64 = a.d % 64 == 0;
    if (a.d_h == 32) {  // N = 96: 128-column tiles with the tail columns clamped
        if (tall) err = launch_gemm_dma<QP, 128, 128, 32, 2, 2, 4, 2>(qp, units, l_a, 96, st);
        else if (k64) err = launch_gemm_dma<QP, 32, 128, 64, 1, 2, 4>(qp, units, l_a, 96, st);
        else err = launch_gemm_dma<QP, 32, 128, 32, 1, 2, 4>(qp, units, l_a, 96, st);
    } else if (a.d_h == 64) {
        if (tall) err = k64 ? launch_gemm_dma<QP, 128, 192, 64, 2, 2, 3>(qp, units, l_a, 192, st)
                            : launch_gemm_dma<QP, 128, 192, 32, 2, 2, 4>(qp, units, l_a, 192, st);
        // 64-row tiles for mid-sized units (the ViT shape: 384 units of 56 rows): three 16 KB stage
        // buffers, so that two workgroups share a CU and the 384 of them run in one round (with
        // 64-deep K-steps and one workgroup per CU the second round ran half empty: SMHA stage 50 -> 46 us)
        else if (k64 && l_a > 32 && (long)units * ((l_a + 63) / 64) >= 256)
            err = launch_gemm_dma<QP, 64, 192, 32, 2, 2, 3, 2>(qp, units, l_a, 192, st);
        // fewer row tiles than compute units: one workgroup per projection (64 columns), three
        // times the workgroups for three reads of the gathered rows out of L2 (the LM shape: 128 row
        // tiles, the stage 26 -> 22.4 us)
        else if (k64 && (long)units * ((l_a + 31) / 32) < 256)
            err = launch_gemm_dma<QP, 32, 64, 64, 1, 2, 4>(qp, units, l_a, 192, st);
        else if (k64) err = launch_gemm_dma<QP, 32, 192, 64, 1, 2, 4>(qp, units, l_a, 192, st);
        else err = launch_gemm_dma<QP, 32, 192, 32, 1, 2, 4>(qp, units, l_a, 192, st);
    } else {
        err = launch_gemm_dma<QP, 128, 128, 32, 2, 2, 4, 2>(qp, units, l_a, 3 * a.d_h, st);
    }
    if (err != hipSuccess) return err;
    return launch_rope<bf16_t>(a, st);
    };
    if (!(a.skip & SMHA_STEP_QKV) && (err = projections()) != hipSuccess) return err;
    if (a.skip & SMHA_STEP_ATTENTION) return hipSuccess;
    return mfma_attn ? launch_attention_mfma(a, st) : launch_attention_generic<bf16_t>(a, st);
}

hipError_t launch_smha_qkv_attention(const SmhaArgs &a, hipStream_t st) { return smha_mfma_qkv_attention(a, st); }

// MFMA path: bf16 storage, d and d_h multiples of 32 (the K segments of the two projections)
static hipError_t smha_mfma(const SmhaArgs &a, hipStream_t st)
{
    typedef OutProjProblem<bf16_t> OP;
    const int l_p = a.l / a.m;
    hipError_t err;
    // the pipelined out-projection finds each patch's segments itself; the other engines read the
    // inverse map
    const bool out_dma = (long)a.k * a.c < (1L << 20);
    if ((err = smha_mfma_qkv_attention(a, st)) != hipSuccess) return err;
    if (a.skip & SMHA_STEP_OUT) return hipSuccess;
    if (!out_dma && (err = launch_inverse_map(a, st)) != hipSuccess) return err;
    // the MFMA kernel addresses one unit's keys with 32-bit element offsets
    const bool mfma_attn = (a.d_h == 32 || a.d_h == 64 || a.d_h == 128) && (long)a.c * l_p * a.d_h < (1L << 31);

    OP op = make_outproj<bf16_t>(a);
    op.once = stream_once((size_t)a.b * a.l * a.d * sizeof(bf16_t));
    if (mfma_attn) {  // the MFMA attention kernel writes o as a (hi, lo) bf16 pair
        op.o_lo = static_cast<const bf16_t *>(a.o_lo);
        op.parts = 2;
    }
    if (!out_dma) {  // segment context of the pipelined engine would not fit
        if (l_p <= 32) return launch_gemm_mfma<OP, 32, 128, 32, 1, 4>(op, a.b * a.m, l_p, a.d, st);
        return launch_gemm_mfma<OP, 64, 128, 32, 2, 2>(op, a.b * a.m, l_p, a.d, st);
    }
    return launch_outproj_dma(op, a.b * a.m, l_p, a.d, st);
}

// ---------------------------------------------------------------------------------------------
// UoME with patch-wise data selection (Eq. 37-40).  Same skeleton as SMHA without the attention:
// first layer per active unit on its gathered rows (UomeDsUpProblem), second layer + index add as
// the output-stationary contraction over the experts that picked each patch (OutProjProblem with
// A^O in the place of W^o and the hidden activations in the place of o).
template <typename T> static UomeDsUpProblem<T> make_ds_up(const UomeDsArgs &a)
{
    UomeDsUpProblem<T> up;
    up.u = static_cast<const T *>(a.u);
    up.a_in = static_cast<const T *>(a.a_in);
    up.expert_idx = a.expert_idx;
    up.patch_idx = a.patch_idx;
    up.expert_gate = (a.flags & F_GATE_EXPERT) ? a.expert_gate : nullptr;
    up.patch_gate = (a.flags & F_GATE_PATCH) ? a.patch_gate : nullptr;
    up.hidden = static_cast<T *>(a.hidden);
    up.l = a.l; up.d = a.d; up.n = a.n; up.kact = a.k; up.m = a.m; up.c = a.c;
    up.l_p = a.l / a.m; up.l_a = a.c * up.l_p; up.d_e = a.d_e;
    return up;
}

template <typename T> static OutProjProblem<T> make_ds_down(const UomeDsArgs &a)
{
    OutProjProblem<T> op;
    op.o = static_cast<const T *>(a.hidden);
    op.o_lo = nullptr;
    op.parts = 1;
    op.wo = static_cast<const T *>(a.a_out);
    op.x = static_cast<const T *>(a.u);
    op.expert_idx = a.expert_idx;
    op.patch_idx = a.patch_idx;
    op.inv_cnt = a.inv_cnt;
    op.inv_ent = a.inv_ent;
    op.out = static_cast<T *>(a.out);
    op.l = a.l; op.d = a.d; op.n = a.n; op.kact = a.k; op.m = a.m; op.c = a.c;
    op.l_p = a.l / a.m; op.l_a = a.c * op.l_p; op.d_h = a.d_e; op.flags = a.flags;
    return op;
}

static hipError_t launch_inverse_map_ds(const UomeDsArgs &a, hipStream_t st)
{
    SmhaArgs s{};  // the inverse map only reads the routing fields
    s.expert_idx = a.expert_idx; s.patch_idx = a.patch_idx;
    s.b = a.b; s.n = a.n; s.k = a.k; s.m = a.m; s.c = a.c;
    s.inv_cnt = a.inv_cnt; s.inv_ent = a.inv_ent;
    return launch_inverse_map(s, st);
}

template <typename T> static hipError_t uome_ds_generic(const UomeDsArgs &a, hipStream_t st)
{
    const int l_p = a.l / a.m, l_a = a.c * l_p;
    hipError_t err;
    if ((err = launch_inverse_map_ds(a, st)) != hipSuccess) return err;
    if ((err = launch_gemm_generic<T>(make_ds_up<T>(a), a.b * a.k, l_a, a.d_e, st)) != hipSuccess) return err;
    return launch_gemm_generic<T>(make_ds_down<T>(a), a.b * a.m, l_p, a.d, st);
}

static hipError_t uome_ds_mfma(const UomeDsArgs &a, hipStream_t st)
{
    typedef UomeDsUpProblem<bf16_t> UP;
    typedef OutProjProblem<bf16_t> OP;
    const int l_p = a.l / a.m, l_a = a.c * l_p, units = a.b * a.k;
    hipError_t err;
    const bool out_dma = (long)a.k * a.c < (1L << 20);
    if (!out_dma && (err = launch_inverse_map_ds(a, st)) != hipSuccess) return err;
    const UP up = make_ds_up<bf16_t>(a);
    const long tiles256 = (long)units * ((l_a + 255) / 256) * ((a.d_e + 127) / 128);
    const long tiles128 = (long)units * ((l_a + 127) / 128) * ((a.d_e + 127) / 128);
    if (l_a > 128 && tiles256 >= 512) err = launch_gemm_dma<UP, 256, 128, 32, 2, 2, 3, 2>(up, units, l_a, a.d_e, st);
    else if (l_a > 64 && a.d % 64 == 0 && tiles128 < 256) err = launch_gemm_dma<UP, 64, 128, 64, 2, 2, 3, 2>(up, units, l_a, a.d_e, st);
    else if (l_a > 64) err = a.d % 64 == 0 ? launch_gemm_dma<UP, 128, 128, 64, 2, 2, 2, 2>(up, units, l_a, a.d_e, st)
                                           : launch_gemm_dma<UP, 128, 128, 32, 2, 2, 4, 2>(up, units, l_a, a.d_e, st);
    else err = launch_gemm_mfma<UP, 64, 64, 32, 2, 2>(up, units, l_a, a.d_e, st);
    if (err != hipSuccess) return err;
    OP op = make_ds_down<bf16_t>(a);
    op.once = stream_once((size_t)a.b * a.l * a.d * sizeof(bf16_t));   // u's last use, the block's output
    if (!out_dma) {
        if (l_p <= 32) return launch_gemm_mfma<OP, 32, 128, 32, 1, 4>(op, a.b * a.m, l_p, a.d, st);
        return launch_gemm_mfma<OP, 64, 128, 32, 2, 2>(op, a.b * a.m, l_p, a.d, st);
    }
    return launch_outproj_dma(op, a.b * a.m, l_p, a.d, st);
}

hipError_t launch_uome_ds(const UomeDsArgs &a, bool bf16, hipStream_t st)
{
    if (bf16 && a.d % 32 == 0 && a.d_e % 32 == 0) return uome_ds_mfma(a, st);
    return bf16 ? uome_ds_generic<bf16_t>(a, st) : uome_ds_generic<float>(a, st);
}

hipError_t launch_smha(const SmhaArgs &a, bool bf16, hipStream_t st)
{
    if (bf16 && a.d % 32 == 0 && a.d_h % 32 == 0) return smha_mfma(a, st);
    return bf16 ? smha_generic<bf16_t>(a, st) : smha_generic<float>(a, st);
}

}  // namespace uoe

// The four contractions of the layer, each stated as a grouped GEMM "problem":
// for a group g, C[M(g), N] = A[M(g), K(g)] * B[K(g), N] with an epilogue, where the rows of A and
// the rows/columns of B are resolved through the routing indices.  A problem is a small POD
// passed by value to a GEMM engine; engines ask it for
//   rows(g), kdim(g), ncols()            problem extents
//   kseg()                               length of one K segment (one expert's slice, or all of K)
//   a_seg_ptr(g, m, seg)   pointer to A[m][seg*kseg]; the segment's kseg elements are contiguous
//   b_seg_ptr(g, seg, nn)  pointer to B[seg*kseg][nn..nn+8)  (nn % 8 == 0)
//   b_stride()             elements between consecutive K rows of B inside a segment
//   col_ctx(g, nn)   whatever the epilogue needs that depends on the column only
//   store(g, m, nn, v, ctx) epilogue for one element
// and, for the MFMA engines (which write 16-byte pieces of output rows),
//   kColScale / col_scale(g, nn)  a per-column factor (constant over 8-column groups), fetched
//                                 once per tile before the K loop
//   epi(v, scale)                 per-element math
//   kRowScale / row_scale(g, m)   a per-row factor, fetched once per tile before the K loop; the
//                                 epilogue passes col_scale * row_scale to epi
//   has_residual() / res8(g, m, nn)  the 16-byte piece of the residual row, loaded in batches
//   put8(g, m, nn, piece)         plain store of a finished piece
//   once, res8_as<ONCE> / put8_as<ONCE>  (optional) a problem with a `once` member lets the launch choose the
//                                 non-temporal versions of the two accesses above, for outputs and
//                                 residuals that this call touches exactly once and that are too large
//                                 for the caches
// and, for the pipelined engine (which may not touch global memory through the compiler inside
// its K loop),
//   seg_ctx(g, seg)               32 bits of routing context of a K segment, looked up once per tile
//   a_ptr_ctx / b_ptr_ctx         a_seg_ptr / b_seg_ptr computed from that context, no lookups
//   kPrepare / prepare(g, segtab, tid, nthreads)  the workgroup builds its segment list itself and
//                                 returns K (out-projection: which experts picked this patch)
// K and N are concatenations of per-expert segments of length `width`; since width % 8 == 0 an
// 8-element run never straddles two experts.
#pragma once
#include "common.h"

namespace uoe {

// 8 bf16 (one 16-byte piece of an output row) + 8 bf16 of a residual row, added in fp32
__device__ __forceinline__ uint4 add8_bf16(uint4 v, uint4 r)
{
    const uint32_t a[4] = {v.x, v.y, v.z, v.w}, b[4] = {r.x, r.y, r.z, r.w};
    uint32_t o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float lo = __uint_as_float(a[i] << 16) + __uint_as_float(b[i] << 16);
        const float hi = __uint_as_float(a[i] & 0xFFFF0000u) + __uint_as_float(b[i] & 0xFFFF0000u);
        o[i] = (uint32_t)f32_to_bf16_bits(lo) | ((uint32_t)f32_to_bf16_bits(hi) << 16);
    }
    return make_uint4(o[0], o[1], o[2], o[3]);
}

// ---------------------------------------------------------------------------------------------
// SMHA Eq. 28-30 with the index selection of Eq. 18 folded into the A-row lookup.
// group = active unit (b, slot s); M = l_a; K = d; N = 3*d_h laid out [q | k | v].
// F32: the single-projection form (nout = 1) stores fp32 rows into q32 instead.
template <typename T, bool F32 = false> struct QkvProblem {
    const T *x, *wq, *wk, *wv;
    const int32_t *expert_idx, *patch_idx;
    T *q, *k, *v;  // [units, l_a, d_h]
    float *q32;    // [units, l_a, d_h] (F32 only)
    static constexpr bool kF32Out = F32;
    __device__ void put4_f32(int g, int r, int nn, float4 val) const
    {
        *reinterpret_cast<float4 *>(q32 + ((size_t)g * l_a + r) * d_h + nn) = val;
    }
    int l, d, n, kact, m, c, l_p, l_a, d_h;
    float q_scale;  // folded into q on the way out (1 for the plain layout)
    int nout;       // 3: q, k and v; 1: the first projection only (N = d_h)
    int v_f16 = 0;  // MFMA engines, bf16 storage: v is written as fp16 (what the attention kernel's P V product takes)
    __device__ bool f16_col(int nn) const { return v_f16 && nn >= 2 * d_h; }

    __device__ int rows(int) const { return l_a; }
    __device__ int kdim(int) const { return d; }
    __device__ int ncols() const { return nout * d_h; }
    __device__ int expert(int g) const { return clampi(expert_idx[g], n); }
    __device__ int token(int g, int r) const
    {
        const int bb = g / kact;
        const int i = expert(g);
        const int t = r / l_p;
        return clampi(patch_idx[((size_t)bb * n + i) * c + t], m) * l_p + (r - t * l_p);
    }
    __device__ int kseg() const { return d; }
    __device__ long b_stride() const { return d_h; }
    __device__ const T *a_seg_ptr(int g, int r, int) const
    {
        const int bb = g / kact;
        return x + ((size_t)bb * l + token(g, r)) * d;
    }
    __device__ const T *b_seg_ptr(int g, int, int nn) const
    {
        const int i = expert(g);
        const int which = nn / d_h, col = nn - which * d_h;
        const T *w = which == 0 ? wq : (which == 1 ? wk : wv);
        return w + (size_t)i * d * d_h + col;
    }
    struct ColCtx {
        int which, col;
    };
    __device__ ColCtx col_ctx(int, int nn) const
    {
        ColCtx cc;
        cc.which = nn / d_h;
        cc.col = nn - cc.which * d_h;
        return cc;
    }
    __device__ void store(int g, int r, int, float val, const ColCtx &cc) const
    {
        if (cc.which == 0) q[((size_t)g * l_a + r) * d_h + cc.col] = from_f32<T>(val * q_scale);
        else if (cc.which == 1) k[((size_t)g * l_a + r) * d_h + cc.col] = from_f32<T>(val);
        else v[((size_t)g * l_a + r) * d_h + cc.col] = from_f32<T>(val);
    }
    // pipelined engine: K is one segment, rows and columns are resolved once before the loop
    __device__ uint32_t seg_ctx(int, int) const { return 0; }
    __device__ const T *a_ptr_ctx(int g, int r, int seg, uint32_t) const { return a_seg_ptr(g, r, seg); }
    __device__ const T *b_ptr_ctx(int g, int seg, int nn, uint32_t) const { return b_seg_ptr(g, seg, nn); }
    // vector epilogue (MFMA engines)
    static constexpr bool kPrepare = false;
    static constexpr bool kRowScale = false;
    static constexpr bool kColScale = true;
    __device__ float col_scale(int, int nn) const { return nn < d_h ? q_scale : 1.0f; }
    __device__ float epi(float val, float scale) const { return val * scale; }
    __device__ bool has_residual() const { return false; }
    __device__ uint4 res8(int, int, int) const { return make_uint4(0, 0, 0, 0); }
    __device__ void put8(int g, int r, int nn, uint4 piece) const
    {
        const int which = nn / d_h, col = nn - which * d_h;
        T *o = which == 0 ? q : (which == 1 ? k : v);
        *reinterpret_cast<uint4 *>(o + ((size_t)g * l_a + r) * d_h + col) = piece;
    }
};

// ---------------------------------------------------------------------------------------------
// SMHA Eq. 35 + Eq. 36, output-stationary: group = (b, patch p); M = l_p; N = d;
// K = (number of active experts that picked p) * d_h.  The per-expert products o_i W^o_i that land
// on the same patch are summed as one contraction over the concatenated K, so each output row is
// written exactly once (residual added in the epilogue) and no atomics are needed.
// o already carries the gate weight of its row.  In the bf16 MFMA path o arrives as two bf16
// buffers, o = hi + lo, so that the attention output enters this contraction with ~16 significant
// bits instead of 8 (the rows of W^o are simply visited twice).
template <typename T> struct OutProjProblem {
    bool once = false;   // this launch streams its output (and residual) past the caches: see store16, wave_write_out
    const T *o, *o_lo, *wo, *x;
    const int32_t *expert_idx, *patch_idx, *inv_cnt, *inv_ent;  // inv_*: engines without prepare()
    T *out;
    int l, d, n, kact, m, c, l_p, l_a, d_h;
    int parts;  // 1: o only; 2: o is a (hi, lo) pair of buffers, contracted as [hi | lo] x [W^o ; W^o]
    uint32_t flags;

    __device__ int rows(int) const { return l_p; }
    __device__ int kdim(int g) const { return inv_cnt[g] * parts * d_h; }
    __device__ int ncols() const { return d; }
    __device__ int kseg() const { return d_h; }
    __device__ long b_stride() const { return d; }
    __device__ const T *a_seg_ptr(int g, int r, int seg) const
    {
        const int bb = g / m;
        const int e = clampi(parts == 2 ? seg >> 1 : seg, kact);
        const T *src = (parts == 2 && (seg & 1)) ? o_lo : o;
        const int ent = clampi(inv_ent[(size_t)g * kact + e], kact * c);  // slot s * c + pick t
        const int s = ent / c, t = ent - s * c;
        return src + (((size_t)bb * kact + s) * l_a + t * l_p + r) * d_h;
    }
    __device__ const T *b_seg_ptr(int g, int seg, int nn) const
    {
        const int bb = g / m;
        const int e = clampi(parts == 2 ? seg >> 1 : seg, kact);
        const int s = clampi(inv_ent[(size_t)g * kact + e], kact * c) / c;
        const int i = clampi(expert_idx[bb * kact + s], n);
        return wo + (size_t)i * d_h * d + nn;
    }
    typedef int ColCtx;
    __device__ ColCtx col_ctx(int, int) const { return 0; }
    __device__ void store(int g, int r, int nn, float val, const ColCtx &) const
    {
        const int bb = g / m, p = g - bb * m;
        const size_t at = ((size_t)bb * l + p * l_p + r) * d + nn;
        if (flags & F_RESIDUAL) val += to_f32(x[at]);
        out[at] = from_f32<T>(val);
    }
    // pipelined engine: per K segment, (slot*c + pick) in bits 0-19, the expert in bits 20-25 and the
    // hi/lo part in bit 26 (needs kact*c < 2^20).  The workgroup builds the list of its group's
    // segments itself (prepare), straight from the routing indices: thread (slot s, pick t) looks
    // whether slot s picked this patch (at most one t per slot does), then the slots that did are
    // listed in slot order, which fixes the summation order.  Returns K; ends on a barrier.
    static constexpr bool kPrepare = true;
    static constexpr bool kRowScale = false;
    __device__ int prepare(int g, uint32_t *segtab, int tid, int nthreads) const
    {
        __shared__ int slot_t[32], slot_e[32];
        const int bb = g / m, pp = g - bb * m;
        if (tid < kact) slot_t[tid] = -1;
        __syncthreads();
        for (int idx = tid; idx < kact * c; idx += nthreads) {
            const int s = idx / c, t = idx - s * c;
            const int i = clampi(expert_idx[bb * kact + s], n);
            if (t == 0) slot_e[s] = i;
            if (clampi(patch_idx[((size_t)bb * n + i) * c + t], m) == pp) slot_t[s] = t;
        }
        __syncthreads();
        int cnt = 0;
        for (int s = 0; s < kact; ++s) {  // every thread walks the (at most 32) slots: cnt is uniform
            const int t = slot_t[s];
            if (t < 0) continue;
            if (tid == 0)
                for (int part = 0; part < parts; ++part)
                    segtab[cnt * parts + part] = (uint32_t)(s * c + t) | ((uint32_t)slot_e[s] << 20) | ((uint32_t)part << 26);
            ++cnt;
        }
        __syncthreads();
        return cnt * parts * d_h;
    }
    __device__ uint32_t seg_ctx(int g, int seg) const
    {
        const int bb = g / m;
        const int e = clampi(parts == 2 ? seg >> 1 : seg, kact);
        const int ent = clampi(inv_ent[(size_t)g * kact + e], kact * c);
        const int i = clampi(expert_idx[bb * kact + ent / c], n);
        return (uint32_t)ent | ((uint32_t)i << 20) | ((parts == 2 && (seg & 1)) ? 1u << 26 : 0u);
    }
    __device__ const T *a_ptr_ctx(int g, int r, int, uint32_t ctx) const
    {
        const int bb = g / m;
        const int ent = (int)(ctx & 0xFFFFFu);
        const int s = ent / c, t = ent - s * c;
        const T *src = (ctx >> 26) & 1u ? o_lo : o;
        return src + (((size_t)bb * kact + s) * l_a + t * l_p + r) * d_h;
    }
    __device__ const T *b_ptr_ctx(int, int, int nn, uint32_t ctx) const { return wo + (size_t)((ctx >> 20) & 0x3Fu) * d_h * d + nn; }
    static constexpr bool kColScale = false;
    __device__ float col_scale(int, int) const { return 1.0f; }
    __device__ float epi(float val, float) const { return val; }
    __device__ size_t at8(int g, int r, int nn) const
    {
        const int bb = g / m, p = g - bb * m;
        return ((size_t)bb * l + p * l_p + r) * d + nn;
    }
    __device__ bool has_residual() const { return flags & F_RESIDUAL; }
    __device__ uint4 res8(int g, int r, int nn) const { return res8_as<false>(g, r, nn); }
    __device__ void put8(int g, int r, int nn, uint4 piece) const { put8_as<false>(g, r, nn, piece); }
    // ONCE: the residual is this tensor's last use in the call and every output piece is written once
    template <bool ONCE> __device__ uint4 res8_as(int g, int r, int nn) const { return load16<ONCE>(x + at8(g, r, nn)); }
    template <bool ONCE> __device__ void put8_as(int g, int r, int nn, uint4 piece) const { store16<ONCE>(out + at8(g, r, nn), piece); }
};

// ---------------------------------------------------------------------------------------------
// UoME Eq. 38: group = sample b; M = l; K = d; N = k*d_e (the sample's active experts side by
// side); epilogue SiLU and the expert's gate.
template <typename T, bool RAW = false> struct UomeUpProblem {
    bool once = false;   // this launch streams its output (and residual) past the caches: see store16, wave_write_out
    const T *u, *a_in;
    const int32_t *expert_idx;
    const float *expert_gate;  // NULL: weight 1
    T *hidden;                 // [b, l, k*d_e]
    int l, d, n, kact, d_e;
    static constexpr bool raw = RAW;   // true: store the plain product (backward pass), no SiLU, no gate

    __device__ int rows(int) const { return l; }
    __device__ int kdim(int) const { return d; }
    __device__ int ncols() const { return kact * d_e; }
    __device__ int kseg() const { return d; }
    __device__ long b_stride() const { return d_e; }
    __device__ const T *a_seg_ptr(int g, int r, int) const { return u + ((size_t)g * l + r) * d; }
    __device__ const T *b_seg_ptr(int g, int, int nn) const
    {
        const int s = nn / d_e;
        const int i = clampi(expert_idx[g * kact + s], n);
        return a_in + (size_t)i * d * d_e + (nn - s * d_e);
    }
    // pipelined engine: no per-segment lookups (K is one segment; the column's expert is resolved
    // once, before the loop)
    __device__ uint32_t seg_ctx(int, int) const { return 0; }
    __device__ const T *a_ptr_ctx(int g, int r, int seg, uint32_t) const { return a_seg_ptr(g, r, seg); }
    __device__ const T *b_ptr_ctx(int g, int seg, int nn, uint32_t) const { return b_seg_ptr(g, seg, nn); }
    typedef float ColCtx;  // the gate of the column's expert
    __device__ ColCtx col_ctx(int g, int nn) const
    {
        if (!expert_gate || raw) return 1.0f;
        return expert_gate[(size_t)g * n + clampi(expert_idx[g * kact + nn / d_e], n)];
    }
    __device__ void store(int g, int r, int nn, float val, const ColCtx &gate) const
    {
        hidden[((size_t)g * l + r) * ((size_t)kact * d_e) + nn] = from_f32<T>(raw ? val : silu(val) * gate);
    }
    static constexpr bool kPrepare = false;
    static constexpr bool kRowScale = false;
    static constexpr bool kColScale = true;
    __device__ float col_scale(int g, int nn) const { return col_ctx(g, nn); }
    __device__ float epi(float val, float gate) const { return raw ? val : silu_fast(val) * gate; }
    __device__ bool has_residual() const { return false; }
    __device__ uint4 res8(int, int, int) const { return make_uint4(0, 0, 0, 0); }
    __device__ void put8(int g, int r, int nn, uint4 piece) const { put8_as<false>(g, r, nn, piece); }
    template <bool ONCE> __device__ uint4 res8_as(int, int, int) const { return make_uint4(0, 0, 0, 0); }
    template <bool ONCE> __device__ void put8_as(int g, int r, int nn, uint4 piece) const   // ONCE: 134 MB on the largest shape, streamed past L2
    {
        store16<ONCE>(hidden + ((size_t)g * l + r) * ((size_t)kact * d_e) + nn, piece);
    }
};

// UoME with patch-wise data selection, first layer (Eq. 37-38): group = active unit (b, slot s);
// M = l_a rows gathered through the unit's patch indices (Eq. 18 folded into the A-row lookup, as
// for QKV); K = d; N = d_e.  Epilogue: SiLU, times the weight of the row's contribution (expert
// gate and/or the gate of the row's patch): the second layer is linear, so the weight can ride on
// the hidden activations and the output-stationary second GEMM needs no per-segment scale.
template <typename T> struct UomeDsUpProblem {
    const T *u, *a_in;
    const int32_t *expert_idx, *patch_idx;
    const float *expert_gate, *patch_gate;  // NULL: weight 1
    T *hidden;                              // [units, l_a, d_e]
    int l, d, n, kact, m, c, l_p, l_a, d_e;

    __device__ int rows(int) const { return l_a; }
    __device__ int kdim(int) const { return d; }
    __device__ int ncols() const { return d_e; }
    __device__ int kseg() const { return d; }
    __device__ long b_stride() const { return d_e; }
    __device__ int expert(int g) const { return clampi(expert_idx[g], n); }
    __device__ int patch(int g, int r) const
    {
        return clampi(patch_idx[((size_t)(g / kact) * n + expert(g)) * c + r / l_p], m);
    }
    __device__ const T *a_seg_ptr(int g, int r, int) const
    {
        return u + ((size_t)(g / kact) * l + patch(g, r) * l_p + r % l_p) * d;
    }
    __device__ const T *b_seg_ptr(int g, int, int nn) const { return a_in + (size_t)expert(g) * d * d_e + nn; }
    __device__ float row_scale(int g, int r) const
    {
        const int bb = g / kact, i = expert(g);
        float w = expert_gate ? expert_gate[(size_t)bb * n + i] : 1.0f;
        if (patch_gate) w *= patch_gate[((size_t)bb * n + i) * m + patch(g, r)];
        return w;
    }
    typedef int ColCtx;
    __device__ ColCtx col_ctx(int, int) const { return 0; }
    __device__ void store(int g, int r, int nn, float val, const ColCtx &) const
    {
        hidden[((size_t)g * l_a + r) * d_e + nn] = from_f32<T>(silu(val) * row_scale(g, r));
    }
    __device__ uint32_t seg_ctx(int, int) const { return 0; }
    __device__ const T *a_ptr_ctx(int g, int r, int seg, uint32_t) const { return a_seg_ptr(g, r, seg); }
    __device__ const T *b_ptr_ctx(int g, int seg, int nn, uint32_t) const { return b_seg_ptr(g, seg, nn); }
    static constexpr bool kPrepare = false;
    static constexpr bool kRowScale = true;
    static constexpr bool kColScale = false;
    __device__ float col_scale(int, int) const { return 1.0f; }
    __device__ float epi(float val, float w) const { return silu_fast(val) * w; }
    __device__ bool has_residual() const { return false; }
    __device__ uint4 res8(int, int, int) const { return make_uint4(0, 0, 0, 0); }
    __device__ void put8(int g, int r, int nn, uint4 piece) const
    {
        *reinterpret_cast<uint4 *>(hidden + ((size_t)g * l_a + r) * d_e + nn) = piece;
    }
};

// UoME Eq. 39 + Eq. 40: group = sample b; M = l; K = k*d_e (row slices of A^O of the active
// experts stacked); N = d; epilogue adds the residual.  One write per output element.
template <typename T> struct UomeDownProblem {
    bool once = false;   // this launch streams its output (and residual) past the caches: see store16, wave_write_out
    const T *hidden, *a_out, *u;
    const int32_t *expert_idx;
    T *out;
    int l, d, n, kact, d_e;
    uint32_t flags;

    __device__ int rows(int) const { return l; }
    __device__ int kdim(int) const { return kact * d_e; }
    __device__ int ncols() const { return d; }
    __device__ int kseg() const { return d_e; }
    __device__ long b_stride() const { return d; }
    __device__ const T *a_seg_ptr(int g, int r, int seg) const
    {
        return hidden + ((size_t)g * l + r) * ((size_t)kact * d_e) + (size_t)clampi(seg, kact) * d_e;
    }
    __device__ const T *b_seg_ptr(int g, int seg, int nn) const
    {
        const int i = clampi(expert_idx[g * kact + clampi(seg, kact)], n);
        return a_out + (size_t)i * d_e * d + nn;
    }
    // pipelined engine: the segment's expert, looked up once before the loop
    __device__ uint32_t seg_ctx(int g, int seg) const { return (uint32_t)clampi(expert_idx[g * kact + clampi(seg, kact)], n); }
    __device__ const T *a_ptr_ctx(int g, int r, int seg, uint32_t) const { return a_seg_ptr(g, r, seg); }
    __device__ const T *b_ptr_ctx(int, int, int nn, uint32_t i) const { return a_out + (size_t)i * d_e * d + nn; }
    typedef int ColCtx;
    __device__ ColCtx col_ctx(int, int) const { return 0; }
    __device__ void store(int g, int r, int nn, float val, const ColCtx &) const
    {
        const size_t at = ((size_t)g * l + r) * d + nn;
        if (flags & F_RESIDUAL) val += to_f32(u[at]);
        out[at] = from_f32<T>(val);
    }
    static constexpr bool kPrepare = false;
    static constexpr bool kRowScale = false;
    static constexpr bool kColScale = false;
    __device__ float col_scale(int, int) const { return 1.0f; }
    __device__ float epi(float val, float) const { return val; }
    __device__ bool has_residual() const { return flags & F_RESIDUAL; }
    __device__ uint4 res8(int g, int r, int nn) const { return res8_as<false>(g, r, nn); }
    __device__ void put8(int g, int r, int nn, uint4 piece) const { put8_as<false>(g, r, nn, piece); }
    // ONCE: u's last use and the block's output
    template <bool ONCE> __device__ uint4 res8_as(int g, int r, int nn) const { return load16<ONCE>(u + ((size_t)g * l + r) * d + nn); }
    template <bool ONCE> __device__ void put8_as(int g, int r, int nn, uint4 piece) const { store16<ONCE>(out + ((size_t)g * l + r) * d + nn, piece); }
};

// ---------------------------------------------------------------------------------------------
// Weight gradients of the backward passes, as split contractions over the tokens with fp32 partial
// tiles.  A launch covers up to four gradient tensors ("sets") of the same shape [n][M][N] at once:
// group = (set * n + expert) * splits + part, partial tile [group][M][N]; a reduction kernel adds
// the parts in order.  The left factor of a set is given TRANSPOSED, token-minor (rows are
// K-contiguous like every A operand); the right factor in its natural token-major layout.
//
// Expert-selection UoME: for expert i,
//   dW[M, N] = sum over the (sample b, slot s) pairs with expert_idx[b,s] == i of  L_{b,s}^T R_b
// contracted over the l tokens of the sample.  K segments = the pairs, found by the workgroup itself
// (prepare), in sample order, which fixes the summation order; the token axis is cut into `splits`
// equal ranges, part j contracts range j of every pair.
//   set 0: dA^O_i   [d_e, d]:  left = H^T  [b][k*d_e][l] (rows s*d_e + e of the pair), right = d_out [b][l][d]
//   set 1: dA^I_i^T [d_e, d]:  left = dZ^T [b][k*d_e][l] (the same rows),              right = u     [b][l][d]
template <typename T> struct WgradProblem {
    const T *left_t[2], *right[2];
    const int32_t *expert_idx;
    float *partial;        // [sets*n*splits, M, N]
    int b, l, n, kact, splits;
    int M, N;              // rows and columns of one expert's gradient
    int left_rows;         // rows of one sample in left_t (k*d_e)
    int left_slot_rows;    // rows of one slot (d_e)
    int right_stride;      // elements between token rows of right

    static constexpr bool kF32Out = true;
    __device__ int rows(int) const { return M; }
    __device__ int ncols() const { return N; }
    __device__ int kseg() const { return l / splits; }
    __device__ long b_stride() const { return right_stride; }
    __device__ int kdim(int) const { return 0; }  // prepare() supplies K
    static constexpr bool kPrepare = true;
    // thread bb looks up which slot of sample bb (if any) holds the expert; the samples that do are
    // listed in sample order (b <= 128 = the engine's segment table)
    __device__ int prepare(int g, uint32_t *segtab, int tid, int) const
    {
        __shared__ int slot_of[128];
        const int expert = (g % (n * splits)) / splits;
        if (tid < b) {
            int slot = -1;
            for (int s = 0; s < kact; ++s)
                if (expert_idx[tid * kact + s] == expert) slot = slot < 0 ? s : slot;
            slot_of[tid] = slot;
        }
        __syncthreads();
        int before = 0, cnt = 0;
        for (int bb = 0; bb < b; ++bb) {  // every thread counts: cnt is uniform
            const bool has = slot_of[bb] >= 0;
            before += (has && bb < tid) ? 1 : 0;
            cnt += has ? 1 : 0;
        }
        if (tid < b && slot_of[tid] >= 0) segtab[before] = ((uint32_t)tid << 8) | (uint32_t)slot_of[tid];
        __syncthreads();
        return cnt * (l / splits);
    }
    __device__ uint32_t seg_ctx(int, int) const { return 0; }
    __device__ const T *a_ptr_ctx(int g, int r, int, uint32_t ctx) const
    {
        const int bb = (int)(ctx >> 8), s = (int)(ctx & 0xFFu);
        const T *base = g < n * splits ? left_t[0] : left_t[1];
        return base + ((size_t)bb * left_rows + (size_t)s * left_slot_rows + r) * l + (g % splits) * (l / splits);
    }
    __device__ const T *b_ptr_ctx(int g, int, int nn, uint32_t ctx) const
    {
        const int bb = (int)(ctx >> 8);
        const T *base = g < n * splits ? right[0] : right[1];
        return base + ((size_t)bb * l + (size_t)(g % splits) * (l / splits)) * right_stride + nn;
    }
    static constexpr bool kRowScale = false;
    static constexpr bool kColScale = false;
    __device__ float col_scale(int, int) const { return 1.0f; }
    __device__ float epi(float val, float) const { return val; }
    __device__ bool has_residual() const { return false; }
    __device__ uint4 res8(int, int, int) const { return make_uint4(0, 0, 0, 0); }
    __device__ void put8(int, int, int, uint4) const {}
    __device__ void put4_f32(int g, int r, int nn, float4 v) const
    {
        *reinterpret_cast<float4 *>(partial + ((size_t)g * M + r) * N + nn) = v;
    }
};

// Blocks with patch-wise data selection (SMHA; the data-selected UoME): for expert i,
//   dW[M, d] = sum over the units (b, slot s) of expert i and their c picks t of
//              L^T[unit][M rows][tokens of pick t]  x  R[b][tokens of the picked patch][d]
// i.e. the left factor is a per-unit tensor in token-minor layout [unit][rows][l_a] (the set's M
// rows start at row0 of the unit's rows) and the right factor is a [b, l, d] tensor (x, u or the
// upstream gradient) whose rows are gathered patch by patch (Eq. 18), never copied.  K segments =
// (unit, pick) of l_p tokens, in (sample, pick) order; the list is cut into `splits` consecutive
// parts.
//   SMHA, M = d_h:  sets 0-2: dW^{q,k,v}_i^T, left = [dq|dk|dv]^T [unit][3d_h][l_a] rows set*d_h.., right = x
//                   set 3:    dW^O_i,         left = (gated o)^T  [unit][d_h][l_a],                  right = d_out
//   UoME, M = d_e:  set 0: dA^O_i, left = H^T [unit][d_e][l_a], right = d_out;  set 1: dA^I_i^T, left = dZ^T, right = u
template <typename T> struct SmhaWgradProblem {
    const T *left_t[4], *right[4];
    int unit_rows[4], row0[4];  // rows of one unit in left_t[set]; first row of the set's M rows
    const int32_t *expert_idx, *patch_idx;
    float *partial;             // [sets*n*splits, M, d]
    int b, l, d, n, kact, m, c, l_p, l_a, splits;
    int M;

    static constexpr bool kF32Out = true;
    __device__ int rows(int) const { return M; }
    __device__ int ncols() const { return d; }
    __device__ int kseg() const { return l_p; }
    __device__ long b_stride() const { return d; }
    __device__ int kdim(int) const { return 0; }
    static constexpr bool kPrepare = true;
    // context of a segment: sample in bits 0-6, slot in bits 7-11, pick in bits 12-21, patch in bits 22-31
    __device__ int prepare(int g, uint32_t *segtab, int tid, int nthreads) const
    {
        __shared__ int slot_of[128];
        const int ge = g % (n * splits), expert = ge / splits, part = ge - expert * splits;
        if (tid < b) {
            int slot = -1;
            for (int s = 0; s < kact; ++s)
                if (expert_idx[tid * kact + s] == expert) slot = slot < 0 ? s : slot;
            slot_of[tid] = slot;
        }
        __syncthreads();
        int units = 0;
        for (int bb = 0; bb < b; ++bb) units += slot_of[bb] >= 0 ? 1 : 0;
        const int total = units * c, per = (total + splits - 1) / splits;
        const int first = part * per, last = min(total, first + per);  // this part's segments
        // thread (sample bb, pick t): its position in the full list is (units before bb) * c + t
        for (int idx = tid; idx < b * c; idx += nthreads) {
            const int bb = idx / c, t = idx - bb * c;
            if (slot_of[bb] < 0) continue;
            int before = 0;
            for (int q = 0; q < bb; ++q) before += slot_of[q] >= 0 ? 1 : 0;
            const int pos = before * c + t;
            if (pos < first || pos >= last || pos - first >= 128) continue;
            const int p = clampi(patch_idx[((size_t)bb * n + expert) * c + t], m);
            segtab[pos - first] = (uint32_t)bb | ((uint32_t)slot_of[bb] << 7) | ((uint32_t)t << 12) | ((uint32_t)p << 22);
        }
        __syncthreads();
        return max(0, min(last - first, 128)) * l_p;
    }
    __device__ uint32_t seg_ctx(int, int) const { return 0; }
    __device__ const T *a_ptr_ctx(int g, int r, int, uint32_t ctx) const
    {
        const int bb = (int)(ctx & 0x7Fu), s = (int)((ctx >> 7) & 0x1Fu), t = (int)((ctx >> 12) & 0x3FFu);
        const int set = g / (n * splits);
        return left_t[set] + (((size_t)bb * kact + s) * unit_rows[set] + row0[set] + r) * l_a + (size_t)t * l_p;
    }
    __device__ const T *b_ptr_ctx(int g, int, int nn, uint32_t ctx) const
    {
        const int bb = (int)(ctx & 0x7Fu), p = (int)(ctx >> 22);
        return right[g / (n * splits)] + ((size_t)bb * l + (size_t)p * l_p) * d + nn;
    }
    static constexpr bool kRowScale = false;
    static constexpr bool kColScale = false;
    __device__ float col_scale(int, int) const { return 1.0f; }
    __device__ float epi(float val, float) const { return val; }
    __device__ bool has_residual() const { return false; }
    __device__ uint4 res8(int, int, int) const { return make_uint4(0, 0, 0, 0); }
    __device__ void put8(int, int, int, uint4) const {}
    __device__ void put4_f32(int g, int r, int nn, float4 v) const
    {
        *reinterpret_cast<float4 *>(partial + ((size_t)g * M + r) * d + nn) = v;
    }
};

}  // namespace uoe

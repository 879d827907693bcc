// Backward passes of the SMHA block (Eq. 27-36, Eq. 32 RoPE, the masks of Sec. III-C.3) and of the UoME block
// in expert-selection mode (Eq. 38-40 with Eq. 24-26) for every shape and storage type the matrix-core
// kernels do not take: fp32 storage, head or expert widths and token counts that are not multiples of 32
// (a 14-token patch, a 196-token sequence).  Same formulas as smha_bwd.hip / uome_bwd.hip on the vector ALU.
// The UoME block's contractions run through one small tiled engine (gen_gemm: 64x64 output tile, 16-deep K
// steps through LDS, 4x4 outputs per thread, operands fetched element by element through a functor that does
// the routing lookups); the SMHA block's kernels are one thread per output element with the contraction
// as a loop.  Every sum has a fixed order (no atomics: results do not depend on scheduling).
// Every intermediate lives in fp32 in the workspace, whatever the storage type; the softmax probabilities
// and their gradients are materialised ([units, l_a, l_a]), which is what bounds the sizes this path is
// meant for.  It favours generality over speed.
#include "common.h"

namespace uoe {

namespace {

constexpr int GT = 256;  // threads per block of every kernel here

inline dim3 blocks_for(long total) { return dim3((unsigned)((total + GT - 1) / GT)); }

// ------------------------------------------------------------------------------------------ tiled engine
// C[m][n] = sum over segments, sum over k of A(m,k) B(k,n) for one group g = blockIdx.z.  A functor F gives
//   rows(g), cols(g), nseg(g); seg(g, s, ctx) -> false to skip a segment; klen(ctx);
//   lhs(ctx, g, m, k), rhs(ctx, g, k, n) as fp32; store(g, m, n, sum)
// and says which index is contiguous in memory for each operand (A_K_FAST / B_K_FAST) so that adjacent
// threads fetch adjacent elements.  Segments and K steps are walked in order: fixed summation order.
template <typename F> __global__ __launch_bounds__(GT) void gen_gemm(F f)
{
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float As[BK][BM + 4], Bs[BK][BN + 4];
    const int g = blockIdx.z, M = f.rows(g), N = f.cols(g);
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    if (m0 >= M || n0 >= N) return;   // uniform over the workgroup
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
    const int nseg = f.nseg(g);
    for (int sg = 0; sg < nseg; ++sg) {
        typename F::Ctx ctx;
        if (!f.seg(g, sg, ctx)) continue;   // uniform
        const int K = f.klen(ctx);
        for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = tid + i * GT;
                const int ak = F::A_K_FAST ? e % BK : e / BM, am = F::A_K_FAST ? e / BK : e % BM;
                As[ak][am] = (m0 + am < M && k0 + ak < K) ? f.lhs(ctx, g, m0 + am, k0 + ak) : 0.f;
                const int bk = F::B_K_FAST ? e % BK : e / BN, bn = F::B_K_FAST ? e / BK : e % BN;
                Bs[bk][bn] = (n0 + bn < N && k0 + bk < K) ? f.rhs(ctx, g, k0 + bk, n0 + bn) : 0.f;
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
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (m < M && n < N) f.store(g, m, n, acc[i][j]);
        }
}

template <typename F> hipError_t launch_gen_gemm(const F &f, int groups, int max_rows, int max_cols, hipStream_t st)
{
    if (groups <= 0 || max_rows <= 0 || max_cols <= 0) return hipSuccess;
    hipLaunchKernelGGL((gen_gemm<F>), dim3((max_cols + 63) / 64, (max_rows + 63) / 64, groups), dim3(GT), 0, st, f);
    return hipGetLastError();
}

struct NoCtx {};

// ------------------------------------------------------------------------------------------ UoME
// a.z and a.dh are fp32 [b, l, k*d_e] here: Z then H, dH_raw then dZ.

// Z = u W1_b (second = false) and dH = d_out W2_b^T (second = true): group = sample, [l] x [k*d_e], K = d
template <typename T, bool second> struct GenUomeProj {
    UomeBwdArgs a;
    typedef NoCtx Ctx;
    static constexpr bool A_K_FAST = true, B_K_FAST = second;   // A^I [d][d_e] runs along the columns, A^O [d_e][d] along K
    __device__ int rows(int) const { return a.l; }
    __device__ int cols(int) const { return a.k * a.d_e; }
    __device__ int nseg(int) const { return 1; }
    __device__ bool seg(int, int, Ctx &) const { return true; }
    __device__ int klen(const Ctx &) const { return a.d; }
    __device__ float a_(const T *base, int g, int m, int k) const { return to_f32(base[((size_t)g * a.l + m) * a.d + k]); }
    __device__ float lhs(const Ctx &, int g, int m, int k) const { return a_(static_cast<const T *>(second ? a.d_out : a.u), g, m, k); }
    __device__ float rhs(const Ctx &, int g, int k, int n) const
    {
        const int s = n / a.d_e, e = n - s * a.d_e, i = clampi(a.expert_idx[g * a.k + s], a.n);
        return second ? to_f32(static_cast<const T *>(a.a_out)[((size_t)i * a.d_e + e) * a.d + k])
                      : to_f32(static_cast<const T *>(a.a_in)[((size_t)i * a.d + k) * a.d_e + e]);
    }
    __device__ void store(int g, int m, int n, float v) const
    {
        static_cast<float *>(second ? a.dh : a.z)[((size_t)g * a.l + m) * ((size_t)a.k * a.d_e) + n] = v;
    }
};

// H = SiLU(Z) w, dZ = dH w SiLU'(Z) in place, and d_gate[b, i(s)] = sum dH SiLU(Z): block = (slot, sample),
// each thread a strided subset of the slot's l*d_e elements in index order, then a fixed tree
__global__ __launch_bounds__(GT) void gen_uome_mid(UomeBwdArgs a)
{
    __shared__ float red[GT];
    const int s = blockIdx.x, bb = blockIdx.y, tid = threadIdx.x;
    const bool gated = (a.flags & F_GATE_EXPERT) && a.expert_gate;
    const int i = clampi(a.expert_idx[bb * a.k + s], a.n);
    const float w = gated ? a.expert_gate[(size_t)bb * a.n + i] : 1.0f;
    const long W = (long)a.k * a.d_e, count = (long)a.l * a.d_e;
    float *zb = static_cast<float *>(a.z), *hb = static_cast<float *>(a.dh);
    float part = 0.f;
    for (long q = tid; q < count; q += GT) {
        const long t = q / a.d_e;
        const long at = ((long)bb * a.l + t) * W + (long)s * a.d_e + (q - t * a.d_e);
        const float z = zb[at], dh = hb[at];
        const float sig = 1.0f / (1.0f + expf(-z)), v = z * sig;
        part = fmaf(dh, v, part);
        zb[at] = v * w;
        hb[at] = dh * w * (sig * (1.0f + z * (1.0f - sig)));
    }
    if (!a.d_gate) return;
    red[tid] = part;
    __syncthreads();
    for (int st = GT / 2; st > 0; st >>= 1) {
        if (tid < st) red[tid] += red[tid + st];
        __syncthreads();
    }
    if (s == 0 && tid < a.n) {  // the experts the sample did not select (all of them without the gate flag)
        bool chosen = false;
        for (int q = 0; q < a.k; ++q) chosen |= clampi(a.expert_idx[bb * a.k + q], a.n) == tid;
        if (!chosen || !(a.flags & F_GATE_EXPERT)) a.d_gate[(size_t)bb * a.n + tid] = 0.f;
    }
    if ((a.flags & F_GATE_EXPERT) && tid == 0) a.d_gate[(size_t)bb * a.n + i] = red[0];
}

// d_u = (d_out) + dZ W1_b^T: group = sample, [l] x [d], K = k*d_e (slot s, hidden column e)
template <typename T> struct GenUomeDu {
    UomeBwdArgs a;
    typedef NoCtx Ctx;
    static constexpr bool A_K_FAST = true, B_K_FAST = true;
    __device__ int rows(int) const { return a.l; }
    __device__ int cols(int) const { return a.d; }
    __device__ int nseg(int) const { return 1; }
    __device__ bool seg(int, int, Ctx &) const { return true; }
    __device__ int klen(const Ctx &) const { return a.k * a.d_e; }
    __device__ float lhs(const Ctx &, int g, int m, int kk) const
    {
        return static_cast<const float *>(a.dh)[((size_t)g * a.l + m) * ((size_t)a.k * a.d_e) + kk];
    }
    __device__ float rhs(const Ctx &, int g, int kk, int j) const
    {
        const int s = kk / a.d_e, e = kk - s * a.d_e, i = clampi(a.expert_idx[g * a.k + s], a.n);
        return to_f32(static_cast<const T *>(a.a_in)[((size_t)i * a.d + j) * a.d_e + e]);
    }
    __device__ void store(int g, int m, int j, float v) const
    {
        const size_t at = ((size_t)g * a.l + m) * a.d + j;
        if (a.flags & F_RESIDUAL) v += to_f32(static_cast<const T *>(a.d_out)[at]);
        static_cast<T *>(a.d_u)[at] = from_f32<T>(v);
    }
};

// dA^O_i [d_e, d] = sum H_{b,s}^T d_out_b (weight gradients 0..n-1) and dA^I_i [d, d_e] = sum u_b^T dZ_{b,s}
// (n..2n-1): segments = the (sample, slot) pairs in order, those of other experts skipped; K = the l tokens.
// With a.splits > 1 the pairs are cut into that many contiguous ranges, group = gradient * splits + range,
// each range's tile goes to a.partial in fp32 and gen_uome_dw_reduce adds the ranges in order.
template <typename T> struct GenUomeDw {
    UomeBwdArgs a;
    struct Ctx {
        int bb, s;
    };
    static constexpr bool A_K_FAST = false, B_K_FAST = false;
    __device__ int grad(int g) const { return g / a.splits; }
    __device__ int per_range() const { return (a.b * a.k + a.splits - 1) / a.splits; }
    __device__ bool second(int g) const { return grad(g) >= a.n; }
    __device__ int rows(int g) const { return second(g) ? a.d : a.d_e; }
    __device__ int cols(int g) const { return second(g) ? a.d_e : a.d; }
    __device__ int nseg(int g) const
    {
        const int first = (g - grad(g) * a.splits) * per_range(), left = a.b * a.k - first;
        return left < per_range() ? (left > 0 ? left : 0) : per_range();
    }
    __device__ bool seg(int g, int sgi, Ctx &c) const
    {
        const int sg = (g - grad(g) * a.splits) * per_range() + sgi;
        c.bb = sg / a.k;
        c.s = sg - c.bb * a.k;
        return clampi(a.expert_idx[sg], a.n) == (second(g) ? grad(g) - a.n : grad(g));
    }
    __device__ int klen(const Ctx &) const { return a.l; }
    __device__ float act(const float *buf, const Ctx &c, int t, int e) const
    {
        return buf[((size_t)c.bb * a.l + t) * ((size_t)a.k * a.d_e) + (size_t)c.s * a.d_e + e];
    }
    __device__ float tok(const void *p, const Ctx &c, int t, int j) const
    {
        return to_f32(static_cast<const T *>(p)[((size_t)c.bb * a.l + t) * a.d + j]);
    }
    __device__ float a_(const Ctx &c, int g, int m, int t) const
    {
        return second(g) ? tok(a.u, c, t, m) : act(static_cast<const float *>(a.z), c, t, m);
    }
    __device__ float lhs(const Ctx &c, int g, int m, int t) const { return a_(c, g, m, t); }
    __device__ float rhs(const Ctx &c, int g, int t, int n) const
    {
        return second(g) ? act(static_cast<const float *>(a.dh), c, t, n) : tok(a.d_out, c, t, n);
    }
    __device__ void store(int g, int m, int n, float v) const
    {
        if (a.splits > 1) {   // [2n][splits][d * d_e]: both gradients have d * d_e elements, in their own layouts
            a.partial[(size_t)g * a.d * a.d_e + (size_t)m * cols(g) + n] = v;
            return;
        }
        if (second(g)) static_cast<T *>(a.d_a_in)[((size_t)(g - a.n) * a.d + m) * a.d_e + n] = from_f32<T>(v);
        else static_cast<T *>(a.d_a_out)[((size_t)g * a.d_e + m) * a.d + n] = from_f32<T>(v);
    }
};

// the ranges of gen_gemm<GenUomeDw> added in order: thread = one weight-gradient element
template <typename T> __global__ __launch_bounds__(GT) void gen_uome_dw_reduce(UomeBwdArgs a)
{
    const long per = (long)a.d * a.d_e, total = 2L * a.n * per, idx = (long)blockIdx.x * GT + threadIdx.x;
    if (idx >= total) return;
    const long gi = idx / per, at = idx - gi * per;   // gradient 0..2n-1, element in its layout
    float sum = 0.f;
    for (int sp = 0; sp < a.splits; ++sp) sum += a.partial[((size_t)gi * a.splits + sp) * per + at];
    if (gi >= a.n) static_cast<T *>(a.d_a_in)[(size_t)(gi - a.n) * per + at] = from_f32<T>(sum);
    else static_cast<T *>(a.d_a_out)[(size_t)gi * per + at] = from_f32<T>(sum);
}

// ------------------------------------------------------------------------------------------ SMHA
// fp32 workspace: f.q, f.kk, f.v, f.o and do_raw [units, l_a, d_h]; dqkv [units, l_a, 3*d_h] as [dq | dk | dv];
// probs and dscores [units, l_a, l_a]; rt [units, l_a]; wt [4, n, d*d_h] (transposed weights, see gen_smha_wt).

struct UnitRow {
    int bb, i, tok;
};
__device__ __forceinline__ UnitRow unit_row(const SmhaArgs &f, int g, int r, int l_p)
{
    UnitRow u;
    u.bb = g / f.k;
    u.i = clampi(f.expert_idx[g], f.n);
    const int p = clampi(f.patch_idx[((size_t)u.bb * f.n + u.i) * f.c + r / l_p], f.m);
    u.tok = p * l_p + r % l_p;
    return u;
}

// weight of row r of unit g in the block's output (Eq. 36 with the gate flags)
__device__ __forceinline__ float row_weight(const SmhaBwdArgs &a, int g, int r, int l_p)
{
    const SmhaArgs &f = a.f;
    const int bb = g / f.k, i = clampi(f.expert_idx[g], f.n);
    float w = 1.0f;
    if (a.flags & F_GATE_EXPERT) w *= a.expert_gate[(size_t)bb * f.n + i];
    if (a.flags & F_GATE_PATCH) {
        const int p = clampi(f.patch_idx[((size_t)bb * f.n + i) * f.c + r / l_p], f.m);
        w *= a.patch_gate[((size_t)bb * f.n + i) * f.m + p];
    }
    return w;
}

// Transposed fp32 copies of the block's weights, so that the kernels whose threads run along the model
// dimension (d_x) or along the head dimension (dO) read them with consecutive lanes on consecutive
// addresses: wt[which][i][e][j] = W^{q,k,v}_i[j][e] for which = 0..2, then wt[3][i][j][e] = W^O_i[e][j].
// Thread = one source element (reads in storage order).
template <typename T> __global__ __launch_bounds__(GT) void gen_smha_wt(SmhaBwdArgs a)
{
    const SmhaArgs &f = a.f;
    const long per = (long)f.n * f.d * f.d_h, idx = (long)blockIdx.x * GT + threadIdx.x;
    if (idx >= 4 * per) return;
    const int which = (int)(idx / per);
    const long q = idx - (long)which * per;
    const int i = (int)(q / ((long)f.d * f.d_h));
    const long rem = q - (long)i * f.d * f.d_h;
    const T *src = static_cast<const T *>(which == 0 ? f.wq : which == 1 ? f.wk : which == 2 ? f.wv : f.wo);
    float *dst = a.wt + (long)which * per + (long)i * f.d * f.d_h;
    if (which < 3) {
        const int j = (int)(rem / f.d_h), e = (int)(rem - (long)j * f.d_h);
        dst[(long)e * f.d + j] = to_f32(src[q]);
    } else {
        const int e = (int)(rem / f.d), j = (int)(rem - (long)e * f.d);
        dst[(long)j * f.d_h + e] = to_f32(src[q]);
    }
}

// q, k, v of the gathered rows (Eq. 18, 28-30): thread = (unit, row, head column)
template <typename T> __global__ __launch_bounds__(GT) void gen_smha_qkv(SmhaBwdArgs a)
{
    const SmhaArgs &f = a.f;
    const int l_p = f.l / f.m, l_a = f.c * l_p;
    const long total = (long)f.b * f.k * l_a * f.d_h, idx = (long)blockIdx.x * GT + threadIdx.x;
    if (idx >= total) return;
    const int e = (int)(idx % f.d_h);
    const long ur = idx / f.d_h;
    const int g = (int)(ur / l_a), r = (int)(ur - (long)g * l_a);
    const UnitRow u = unit_row(f, g, r, l_p);
    const T *xr = static_cast<const T *>(f.x) + ((size_t)u.bb * f.l + u.tok) * f.d;
    const size_t wat = (size_t)u.i * f.d * f.d_h + e;
    const T *wq = static_cast<const T *>(f.wq) + wat, *wk = static_cast<const T *>(f.wk) + wat, *wv = static_cast<const T *>(f.wv) + wat;
    float q = 0.f, k = 0.f, v = 0.f;
    for (int j = 0; j < f.d; ++j) {
        const float xv = to_f32(xr[j]);
        q = fmaf(xv, to_f32(wq[(size_t)j * f.d_h]), q);
        k = fmaf(xv, to_f32(wk[(size_t)j * f.d_h]), k);
        v = fmaf(xv, to_f32(wv[(size_t)j * f.d_h]), v);
    }
    static_cast<float *>(f.q)[idx] = q;
    static_cast<float *>(f.kk)[idx] = k;
    static_cast<float *>(f.v)[idx] = v;
}

// Partial RoPE of Eq. 32 on two [units, l_a, stride] fp32 arrays (columns col0.. of each row hold a head), in
// place: pairs (2i, 2i+1) of the last rope_dim dims rotated by row position * 10000^(-2i/rope_dim);
// inverse = the transposed rotation (the gradient's way back).  Thread = (unit row, pair).
__global__ __launch_bounds__(GT) void gen_smha_rope(SmhaArgs f, float *pa, float *pb, int stride, int inverse)
{
    const int l_a = f.c * (f.l / f.m), half = f.rope_dim >> 1;
    const long total = (long)f.b * f.k * l_a * half, idx = (long)blockIdx.x * GT + threadIdx.x;
    if (idx >= total) return;
    const int i = (int)(idx % half);
    const long row = idx / half;
    const int r = (int)(row % l_a);
    const float theta = exp2f(-(2.0f * (float)i / (float)f.rope_dim) * 13.287712379549449f);  // log2(10000)
    float sn, cs;
    sincosf((float)r * theta, &sn, &cs);
    if (inverse) sn = -sn;
    const size_t at = (size_t)row * stride + (f.d_h - f.rope_dim) + 2 * i;
    const float a0 = pa[at], a1 = pa[at + 1], b0 = pb[at], b1 = pb[at + 1];
    pa[at] = a0 * cs - a1 * sn;
    pa[at + 1] = a0 * sn + a1 * cs;
    pb[at] = b0 * cs - b1 * sn;
    pb[at + 1] = b0 * sn + b1 * cs;
}

__device__ __forceinline__ bool gen_key_ok(const SmhaArgs &f, int g, int r, int key, int l_p)
{
    if ((f.flags & F_CAUSAL) && key > r) return false;
    if (!f.pad_mask) return true;
    const UnitRow u = unit_row(f, g, key, l_p);
    return f.pad_mask[(size_t)u.bb * f.l + u.tok] != 0;   // Eq. 41: padded keys are out of every softmax
}

// scaled scores of the admissible (query, key) pairs, -inf elsewhere: thread = (unit, query, key)
__global__ __launch_bounds__(GT) void gen_smha_scores(SmhaBwdArgs a)
{
    const SmhaArgs &f = a.f;
    const int l_p = f.l / f.m, l_a = f.c * l_p;
    const long total = (long)f.b * f.k * l_a * l_a, idx = (long)blockIdx.x * GT + threadIdx.x;
    if (idx >= total) return;
    const int key = (int)(idx % l_a);
    const long ur = idx / l_a;
    const int g = (int)(ur / l_a), r = (int)(ur - (long)g * l_a);
    float s = -INFINITY;
    if (gen_key_ok(f, g, r, key, l_p)) {
        const float *q = static_cast<const float *>(f.q) + ur * f.d_h;
        const float *k = static_cast<const float *>(f.kk) + ((long)g * l_a + key) * f.d_h;
        s = 0.f;
        for (int e = 0; e < f.d_h; ++e) s = fmaf(q[e], k[e], s);
        s *= rsqrtf((float)f.d_h);
    }
    a.probs[idx] = s;
}

// softmax of every query row in place (Eq. 33); a row with no admissible key becomes all zeros
__global__ __launch_bounds__(GT) void gen_smha_softmax(SmhaBwdArgs a)
{
    const SmhaArgs &f = a.f;
    const int l_a = f.c * (f.l / f.m);
    const long total = (long)f.b * f.k * l_a, ur = (long)blockIdx.x * GT + threadIdx.x;
    if (ur >= total) return;
    float *p = a.probs + ur * l_a;
    float mx = -INFINITY;
    for (int j = 0; j < l_a; ++j) mx = fmaxf(mx, p[j]);
    if (mx == -INFINITY) {
        for (int j = 0; j < l_a; ++j) p[j] = 0.f;
        return;
    }
    float den = 0.f;
    for (int j = 0; j < l_a; ++j) den += expf(p[j] - mx);
    const float inv = 1.0f / den;
    for (int j = 0; j < l_a; ++j) p[j] = expf(p[j] - mx) * inv;
}

// o = P v (Eq. 34, no gate): thread = (unit, row, head column)
__global__ __launch_bounds__(GT) void gen_smha_o(SmhaBwdArgs a)
{
    const SmhaArgs &f = a.f;
    const int l_a = f.c * (f.l / f.m);
    const long total = (long)f.b * f.k * l_a * f.d_h, idx = (long)blockIdx.x * GT + threadIdx.x;
    if (idx >= total) return;
    const int e = (int)(idx % f.d_h);
    const long ur = idx / f.d_h;
    const int g = (int)(ur / l_a);
    const float *p = a.probs + ur * l_a, *v = static_cast<const float *>(f.v) + (long)g * l_a * f.d_h + e;
    float o = 0.f;
    for (int j = 0; j < l_a; ++j) o = fmaf(p[j], v[(long)j * f.d_h], o);
    static_cast<float *>(f.o)[idx] = o;
}

// dO_raw = G[T] W^O_i^T: thread = (unit, row, head column)
template <typename T> __global__ __launch_bounds__(GT) void gen_smha_do(SmhaBwdArgs a)
{
    const SmhaArgs &f = a.f;
    const int l_p = f.l / f.m, l_a = f.c * l_p;
    const long total = (long)f.b * f.k * l_a * f.d_h, idx = (long)blockIdx.x * GT + threadIdx.x;
    if (idx >= total) return;
    const int e = (int)(idx % f.d_h);
    const long ur = idx / f.d_h;
    const int g = (int)(ur / l_a), r = (int)(ur - (long)g * l_a);
    const UnitRow u = unit_row(f, g, r, l_p);
    const T *gr = static_cast<const T *>(a.d_out) + ((size_t)u.bb * f.l + u.tok) * f.d;
    const float *wo = a.wt + ((size_t)3 * f.n + u.i) * f.d * f.d_h + e;   // column e of the transposed W^O_i [d][d_h]
    float acc = 0.f;
    for (int j = 0; j < f.d; ++j) acc = fmaf(to_f32(gr[j]), wo[(size_t)j * f.d_h], acc);
    a.do_raw[idx] = acc;
}

// r_t = dO_raw_t . o_t (the gradient of the row's weight), then dO = w dO_raw in place: thread = (unit, row)
__global__ __launch_bounds__(GT) void gen_smha_row(SmhaBwdArgs a)
{
    const SmhaArgs &f = a.f;
    const int l_p = f.l / f.m, l_a = f.c * l_p;
    const long total = (long)f.b * f.k * l_a, ur = (long)blockIdx.x * GT + threadIdx.x;
    if (ur >= total) return;
    const int g = (int)(ur / l_a), r = (int)(ur - (long)g * l_a);
    const float w = row_weight(a, g, r, l_p);
    float *dr = a.do_raw + ur * f.d_h;
    const float *o = static_cast<const float *>(f.o) + ur * f.d_h;
    float dot = 0.f;
    for (int e = 0; e < f.d_h; ++e) {
        dot = fmaf(dr[e], o[e], dot);
        dr[e] *= w;
    }
    a.rt[ur] = dot;
}

// dP = dO V^T: thread = (unit, query, key)
__global__ __launch_bounds__(GT) void gen_smha_dp(SmhaBwdArgs a)
{
    const SmhaArgs &f = a.f;
    const int l_a = f.c * (f.l / f.m);
    const long total = (long)f.b * f.k * l_a * l_a, idx = (long)blockIdx.x * GT + threadIdx.x;
    if (idx >= total) return;
    const int key = (int)(idx % l_a);
    const long ur = idx / l_a;
    const int g = (int)(ur / l_a);
    const float *d_o = a.do_raw + ur * f.d_h, *v = static_cast<const float *>(f.v) + ((long)g * l_a + key) * f.d_h;
    float s = 0.f;
    for (int e = 0; e < f.d_h; ++e) s = fmaf(d_o[e], v[e], s);
    a.dscores[idx] = s;
}

// dS = P * (dP - D), D = sum_j P_j dP_j, in place: thread = (unit, query)
__global__ __launch_bounds__(GT) void gen_smha_ds(SmhaBwdArgs a)
{
    const SmhaArgs &f = a.f;
    const int l_a = f.c * (f.l / f.m);
    const long total = (long)f.b * f.k * l_a, ur = (long)blockIdx.x * GT + threadIdx.x;
    if (ur >= total) return;
    const float *p = a.probs + ur * l_a;
    float *ds = a.dscores + ur * l_a;
    float dsum = 0.f;
    for (int j = 0; j < l_a; ++j) dsum = fmaf(p[j], ds[j], dsum);
    for (int j = 0; j < l_a; ++j) ds[j] = p[j] * (ds[j] - dsum);
}

// dQ = dS K / sqrt(d_h), dK = dS^T Q / sqrt(d_h), dV = P^T dO: thread = (unit, row, head column)
__global__ __launch_bounds__(GT) void gen_smha_dqkv(SmhaBwdArgs a)
{
    const SmhaArgs &f = a.f;
    const int l_a = f.c * (f.l / f.m);
    const long total = (long)f.b * f.k * l_a * f.d_h, idx = (long)blockIdx.x * GT + threadIdx.x;
    if (idx >= total) return;
    const int e = (int)(idx % f.d_h);
    const long ur = idx / f.d_h;
    const int g = (int)(ur / l_a), r = (int)(ur - (long)g * l_a);
    const long ubase = (long)g * l_a;
    const float *q = static_cast<const float *>(f.q) + ubase * f.d_h + e, *k = static_cast<const float *>(f.kk) + ubase * f.d_h + e;
    const float *d_o = a.do_raw + ubase * f.d_h + e;
    const float *ds_row = a.dscores + ur * l_a;            // dS[r, :]
    const float *ds_col = a.dscores + ubase * l_a + r;     // dS[:, r]
    const float *p_col = a.probs + ubase * l_a + r;        // P[:, r]
    float dq = 0.f, dk = 0.f, dv = 0.f;
    for (int j = 0; j < l_a; ++j) {
        dq = fmaf(ds_row[j], k[(long)j * f.d_h], dq);
        dk = fmaf(ds_col[(long)j * l_a], q[(long)j * f.d_h], dk);
        dv = fmaf(p_col[(long)j * l_a], d_o[(long)j * f.d_h], dv);
    }
    const float scale = rsqrtf((float)f.d_h);
    float *out = static_cast<float *>(a.dqkv) + ur * 3 * f.d_h + e;
    out[0] = dq * scale;
    out[f.d_h] = dk * scale;
    out[2 * f.d_h] = dv;
}

// d_x = (G) + sum over the units that picked the token's patch of [dq|dk|dv] [W^q|W^k|W^v]_i^T, slots then
// picks in order: thread = (token, model column j)
template <typename T> __global__ __launch_bounds__(GT) void gen_smha_dx(SmhaBwdArgs a)
{
    const SmhaArgs &f = a.f;
    const int l_p = f.l / f.m, l_a = f.c * l_p;
    const long total = (long)f.b * f.l * f.d, idx = (long)blockIdx.x * GT + threadIdx.x;
    if (idx >= total) return;
    const long trow = idx / f.d;
    const int j = (int)(idx - trow * f.d), bb = (int)(trow / f.l), tok = (int)(trow - (long)bb * f.l);
    const int patch = tok / l_p, within = tok - patch * l_p;
    float acc = (a.flags & F_RESIDUAL) ? to_f32(static_cast<const T *>(a.d_out)[idx]) : 0.f;
    for (int s = 0; s < f.k; ++s) {
        const int g = bb * f.k + s, i = clampi(f.expert_idx[g], f.n);
        const int32_t *picks = f.patch_idx + ((size_t)bb * f.n + i) * f.c;
        const size_t per = (size_t)f.n * f.d * f.d_h;
        const float *wq = a.wt + (size_t)i * f.d_h * f.d + j, *wk = wq + per, *wv = wk + per;   // column j of the transposed [d_h, d] weights
        for (int t = 0; t < f.c; ++t) {
            if (clampi(picks[t], f.m) != patch) continue;
            const float *row = static_cast<const float *>(a.dqkv) + ((long)g * l_a + t * l_p + within) * 3 * f.d_h;
            for (int e = 0; e < f.d_h; ++e) {
                acc = fmaf(row[e], wq[(size_t)e * f.d], acc);
                acc = fmaf(row[f.d_h + e], wk[(size_t)e * f.d], acc);
                acc = fmaf(row[2 * f.d_h + e], wv[(size_t)e * f.d], acc);
            }
        }
    }
    static_cast<T *>(a.d_x)[idx] = from_f32<T>(acc);
}

// dW^{q,k,v}_i [d, d_h] = sum x[T]^T d{Q,K,V} and dW^O_i [d_h, d] = sum (w o)^T G[T] over the units of
// expert i, units then rows in order: thread = four consecutive weight elements (four head columns of one
// row of dW^{q,k,v}, four model columns of one row of dW^O), so that the operand every lane shares is
// loaded once for four products
template <typename T> __global__ __launch_bounds__(GT) void gen_smha_dw(SmhaBwdArgs a)
{
    const SmhaArgs &f = a.f;
    const int l_p = f.l / f.m, l_a = f.c * l_p, units = f.b * f.k;
    const long per = (long)f.n * f.d * f.d_h, quads = per / 4, tid = (long)blockIdx.x * GT + threadIdx.x;
    if (tid >= 4 * quads * a.splits) return;
    // a.splits > 1: the units are cut into that many contiguous ranges, one thread per (range, four elements),
    // partial sums to a.partial [splits][4][per], added in range order by gen_smha_dw_reduce
    const int sp = (int)(tid / (4 * quads));
    const long idx = tid - (long)sp * 4 * quads;
    const int per_range = (units + a.splits - 1) / a.splits;
    const int g_first = sp * per_range, g_end = g_first + per_range < units ? g_first + per_range : units;
    const int which = (int)(idx / quads);   // 0..2: dW^q, dW^k, dW^v; 3: dW^O
    const long q = (idx - (long)which * quads) * 4;   // first of the four elements (d_h and d are multiples of 8)
    const int i = (int)(q / ((long)f.d * f.d_h));
    const long rem = q - (long)i * f.d * f.d_h;
    // which < 3: row j, columns e..e+3 of [d][d_h]; which == 3: row e, columns j..j+3 of [d_h][d]
    const int e = which < 3 ? (int)(rem % f.d_h) : (int)(rem / f.d), j = which < 3 ? (int)(rem / f.d_h) : (int)(rem % f.d);
    const T *tokens = static_cast<const T *>(which < 3 ? f.x : a.d_out);
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int g = g_first; g < g_end; ++g) {
        if (clampi(f.expert_idx[g], f.n) != i) continue;
        const int bb = g / f.k;
        const int32_t *picks = f.patch_idx + ((size_t)bb * f.n + i) * f.c;
        for (int t = 0; t < f.c; ++t) {
            const int p = clampi(picks[t], f.m);
            const T *tk = tokens + ((size_t)bb * f.l + (size_t)p * l_p) * f.d + j;
            const long r0 = (long)g * l_a + t * l_p;
            if (which < 3) {
                for (int rr = 0; rr < l_p; ++rr) {
                    const float4 left = *reinterpret_cast<const float4 *>(static_cast<const float *>(a.dqkv) + (r0 + rr) * 3 * f.d_h + which * f.d_h + e);
                    const float right = to_f32(tk[(size_t)rr * f.d]);
                    acc[0] = fmaf(left.x, right, acc[0]);
                    acc[1] = fmaf(left.y, right, acc[1]);
                    acc[2] = fmaf(left.z, right, acc[2]);
                    acc[3] = fmaf(left.w, right, acc[3]);
                }
            } else {
                const float w = row_weight(a, g, t * l_p, l_p);   // one weight per (unit, pick)
                for (int rr = 0; rr < l_p; ++rr) {
                    const float left = static_cast<const float *>(f.o)[(r0 + rr) * f.d_h + e] * w;
#pragma unroll
                    for (int u = 0; u < 4; ++u) acc[u] = fmaf(left, to_f32(tk[(size_t)rr * f.d + u]), acc[u]);
                }
            }
        }
    }
    if (a.splits > 1) {
        float *part = a.partial + ((size_t)sp * 4 + which) * per + q;
#pragma unroll
        for (int u = 0; u < 4; ++u) part[u] = acc[u];
        return;
    }
    T *dst = static_cast<T *>(which == 0 ? a.d_wq : which == 1 ? a.d_wk : which == 2 ? a.d_wv : a.d_wo);
#pragma unroll
    for (int u = 0; u < 4; ++u) dst[q + u] = from_f32<T>(acc[u]);
}

// the unit ranges of gen_smha_dw added in order: thread = one weight-gradient element
template <typename T> __global__ __launch_bounds__(GT) void gen_smha_dw_reduce(SmhaBwdArgs a)
{
    const SmhaArgs &f = a.f;
    const long per = (long)f.n * f.d * f.d_h, idx = (long)blockIdx.x * GT + threadIdx.x;
    if (idx >= 4 * per) return;
    const int which = (int)(idx / per);
    const long q = idx - (long)which * per;
    float sum = 0.f;
    for (int sp = 0; sp < a.splits; ++sp) sum += a.partial[((size_t)sp * 4 + which) * per + q];
    T *dst = static_cast<T *>(which == 0 ? a.d_wq : which == 1 ? a.d_wk : which == 2 ? a.d_wv : a.d_wo);
    dst[q] = from_f32<T>(sum);
}

template <typename T> hipError_t uome_backward_generic(const UomeBwdArgs &a, hipStream_t st)
{
    const int W = a.k * a.d_e;
    hipError_t err;
    if ((err = launch_gen_gemm(GenUomeProj<T, false>{a}, a.b, a.l, W, st)) != hipSuccess) return err;
    if ((err = launch_gen_gemm(GenUomeProj<T, true>{a}, a.b, a.l, W, st)) != hipSuccess) return err;
    hipLaunchKernelGGL(gen_uome_mid, dim3(a.k, a.b), dim3(GT), 0, st, a);
    if ((err = hipGetLastError()) != hipSuccess) return err;
    if ((err = launch_gen_gemm(GenUomeDu<T>{a}, a.b, a.l, a.d, st)) != hipSuccess) return err;
    if ((err = launch_gen_gemm(GenUomeDw<T>{a}, 2 * a.n * a.splits, a.d > a.d_e ? a.d : a.d_e, a.d > a.d_e ? a.d : a.d_e, st)) != hipSuccess)
        return err;
    if (a.splits > 1) {
        hipLaunchKernelGGL((gen_uome_dw_reduce<T>), blocks_for(2L * a.n * a.d * a.d_e), dim3(GT), 0, st, a);
        err = hipGetLastError();
    }
    return err;
}

template <typename T> hipError_t smha_backward_generic(const SmhaBwdArgs &a, hipStream_t st)
{
    const SmhaArgs &f = a.f;
    const int l_p = f.l / f.m, l_a = f.c * l_p;
    const long rows = (long)f.b * f.k * l_a, elems = rows * f.d_h, pairs = rows * l_a;
    const long rope_pairs = rows * (f.rope_dim >> 1);
    hipError_t err;
#define UOE_GEN(kernel, total, ...)                                                       \
    hipLaunchKernelGGL(kernel, blocks_for(total), dim3(GT), 0, st, __VA_ARGS__);          \
    if ((err = hipGetLastError()) != hipSuccess) return err
    UOE_GEN((gen_smha_wt<T>), 4L * f.n * f.d * f.d_h, a);
    UOE_GEN((gen_smha_qkv<T>), elems, a);
    if (f.rope_dim > 0) { UOE_GEN(gen_smha_rope, rope_pairs, f, static_cast<float *>(f.q), static_cast<float *>(f.kk), f.d_h, 0); }
    UOE_GEN(gen_smha_scores, pairs, a);
    UOE_GEN(gen_smha_softmax, rows, a);
    UOE_GEN(gen_smha_o, elems, a);
    UOE_GEN((gen_smha_do<T>), elems, a);
    UOE_GEN(gen_smha_row, rows, a);
    if ((err = launch_unit_gate_grads(a, st)) != hipSuccess) return err;
    UOE_GEN(gen_smha_dp, pairs, a);
    UOE_GEN(gen_smha_ds, rows, a);
    UOE_GEN(gen_smha_dqkv, elems, a);
    if (f.rope_dim > 0) {
        float *dq = static_cast<float *>(a.dqkv);
        UOE_GEN(gen_smha_rope, rope_pairs, f, dq, dq + f.d_h, 3 * f.d_h, 1);
    }
    UOE_GEN((gen_smha_dx<T>), (long)f.b * f.l * f.d, a);
    UOE_GEN((gen_smha_dw<T>), (long)f.n * f.d * f.d_h * a.splits, a);
    if (a.splits > 1) { UOE_GEN((gen_smha_dw_reduce<T>), 4L * f.n * f.d * f.d_h, a); }
#undef UOE_GEN
    return hipSuccess;
}

}  // namespace

hipError_t launch_uome_backward_generic(const UomeBwdArgs &a, bool bf16, hipStream_t st)
{
    return bf16 ? uome_backward_generic<bf16_t>(a, st) : uome_backward_generic<float>(a, st);
}

hipError_t launch_smha_backward_generic(const SmhaBwdArgs &a, bool bf16, hipStream_t st)
{
    return bf16 ? smha_backward_generic<bf16_t>(a, st) : smha_backward_generic<float>(a, st);
}

}  // namespace uoe

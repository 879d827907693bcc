// Routing of one block (Sec. III-B): expert-selection router (Eq. 21-22) and patch-wise
// data-selection router (Eq. 13, 14, 17).
//
// Kernels:
//   route_expert_mfma : expert router, bf16.  Eq. 21 is a [b, l*d] x [l*d, n] product with a huge
//                       inner dimension: a workgroup owns a chunk of the flat l*d axis for up to
//                       64 samples and all experts, its waves stream x and W_E straight from
//                       global memory into v_mfma_f32_16x16x32_bf16 fragments (rows = samples,
//                       columns = experts).  Every byte of x and of W_E is requested once.
//   route_partial<E>  : expert router on the vector ALU (fp32 storage).  A workgroup owns (chunk
//                       of tokens, sample); each wave streams token rows of x and the matching rows
//                       of the n W_E slices and keeps n running dot products per lane (a W_E chunk
//                       is shared by the b samples through L2).
//   route_data_mfma   : data router, bf16.  t1 = x W_B for 16 tokens per wave as
//                       v_mfma_f32_16x16x32_bf16 (A fragments straight from global, W_B^T staged in
//                       LDS), then the chunk's rows of W_A fold t1 into a partial [n,m] logit tile.
//   route_partial<D>  : the same data router on the vector ALU (fp32 storage, or W_B too large
//                       for LDS next to the MFMA staging).
//   route_reduce      : sums the data router's per-chunk partials in a fixed order (deterministic).
//   route_select      : per (expert row, sample): + noise, softmax over experts (Eq. 14 / 21), then
//                       top-c per expert and top-k per sample by rank counting: rank(j) = #{j' :
//                       g_j' > g_j or (g_j' == g_j and j' < j)}; keep rank < c.  The output slot of
//                       a kept index is the number of kept lower indices, so the list comes out
//                       ascending with no sort and ties go to the lower index by construction.
#include "common.h"
#include <cstdlib>

namespace uoe {

// LDS row pitch in dwords for a [k][cols] bf16 tile read with the transposing LDS read: the four
// 64-byte row pieces a half-wave touches must fall into different banks (pitch % 64 dwords = 16 or 48)
__host__ __device__ constexpr int b_pitch16(int cols)
{
    int p = cols / 2;
    while ((p % 64) != 16 && (p % 64) != 48) p += 4;
    return p;
}

int route_tokens_per_chunk(int b, int l)
{
    // aim for >= ~512 workgroups but keep a chunk within [16, 64] tokens (longer chunks stream
    // better: measured 3.3 / 3.6 / 3.9 TB/s at 16 / 32 / 64 tokens on the largest shape)
    long tc = ((long)b * l) / 512;
    if (tc > l / 8) tc = l / 8;  // at least ~8 chunks per sample so the last, short chunk does not dominate
    tc = (tc / 4) * 4;
    if (tc < 16) tc = 16;
    if (tc > 64) tc = 64;
    if (tc > l) tc = l;
    return (int)tc;
}

// Expert router, MFMA kernel: tokens per chunk.  The chunk count does not depend on b (a workgroup
// takes all samples of its chunk), so aim for ~512 chunks.
int route_expert_mfma_tokens_per_chunk(int b, int l, int d, int n)
{
    (void)b; (void)d; (void)n;  // ~512 chunks whatever the shape: measured best from `lm` to `large`
    const int tc = l / 512;
    return tc < 1 ? 1 : tc;
}

// Data router: tokens per chunk and whether the MFMA kernel applies.  waves*16 tokens per chunk for
// the MFMA kernel, else the expert router's chunking.
static int data_mfma_waves(int, int)
{
    return 4;  // 64 tokens per workgroup: the W_B staging is shared by four waves
}
// LDS of the MFMA data router: W_B as it is, [d][np] in blocks of 8 rows (see the kernel), then t1.
static size_t data_mfma_wb_bytes(int n, int d)
{
    const int np = (n + 15) & ~15;
    return (size_t)((d + 7) / 8) * (8 * np * 2 + (np == 16 ? 128 : 32));
}
static size_t data_mfma_lds(int n, int d, int waves)
{
    const int np = (n + 15) & ~15;
    // W_B, t1 [waves*16][np], and the fold's per-token-group partial sums (at most 8 per thread)
    return data_mfma_wb_bytes(n, d) + (size_t)waves * 16 * np * sizeof(float) + (size_t)waves * 64 * 8 * sizeof(float);
}
bool route_data_uses_mfma(int b, int l, int d, int n, bool bf16)
{
    return bf16 && data_mfma_lds(n, d, data_mfma_waves(b, l)) <= 60 * 1024;
}
// Plan of the streaming router kernel (route_stream_kernel): one workgroup per compute unit, each
// owning a contiguous run of whole tokens.
RouteStreamPlan route_stream_plan(int b, int l, int d, int n, bool bf16, bool has_d)
{
    RouteStreamPlan p{};
    if (!bf16 || d % 128 != 0) return p;   // every wave takes d/128 of the 32-element steps of each token
    p.rt = b > 32 ? 4 : (b > 16 ? 2 : 1);
    p.ct = n <= 16 ? 1 : 2;
    p.rb = p.rt == 1 ? 1024 : 512;
    const int bg = b < p.rt * 16 ? b : p.rt * 16;           // samples of one workgroup
    const int rows = bg + n, rpi = 1024 / p.rb;             // rows per stage; rows per load instruction
    p.ipw = ((rows + rpi - 1) / rpi + 3) / 4;
    p.tpc = (l + ROUTE_STREAM_CHUNKS - 1) / ROUTE_STREAM_CHUNKS;
    p.nchunks = (l + p.tpc - 1) / p.tpc;
    const int np = p.ct * 16;
    p.lds = (size_t)3 * p.ipw * 4 * 1024 + sizeof(float) * 4 * p.rt * 16 * (np + 1);
    if (has_d) p.lds += (size_t)(d / 8) * (8 * np * 2 + (np == 16 ? 128 : 32)) + (size_t)4 * p.tpc * bg * n * sizeof(float);
    p.ok = p.lds <= 150 * 1024 && p.ipw <= 16;
    return p;
}
// Token ranges of route_fold_mfma: whole 128-token blocks (32 per wave and step), at most 512 tokens,
// about 256 workgroups when the batch allows.  Up to 16 ranges per sample route_select adds the
// partial tiles up itself; beyond that route_reduce does.
RouteFoldPlan route_fold_plan(int b, int l)
{
    int want = 256 / b;
    want = want < 1 ? 1 : (want > 16 ? 16 : want);
    RouteFoldPlan p;
    p.tr = ((l + want - 1) / want + 127) / 128 * 128;
    if (p.tr > 512) p.tr = 512;   // 4 steps of 32 tokens per wave: every load of a wave is in flight at once
    p.ranges = (l + p.tr - 1) / p.tr;
    return p;
}

// Whether the streaming kernel is used when it applies: from about 100 MB of x and W_E.  Below that the
// register-staged kernels are as fast or faster (their workgroups are many and short, which suits
// inputs that a single round of 256 long-lived workgroups does not keep busy), measured per shape:
// 50 MB (b16 l4096 d256 n8) runs at 29-30 us either way, 335 MB (b4 l8192 d1024 n16) at 95 vs 113 us.
// UOE_ROUTE_STREAM_MIN_BYTES in the environment overrides the threshold (0: whenever the kernel applies).
bool route_stream_pays(int b, int l, int d, int n)
{
    const char *env = getenv("UOE_ROUTE_STREAM_MIN_BYTES");
    const double min_bytes = env ? atof(env) : 100e6;
    return ((double)b + n) * l * d * 2 >= min_bytes;
}
int route_data_tokens_per_chunk(int b, int l, int d, int n, bool bf16)
{
    if (route_stream_plan(b, l, d, n, bf16, true).ok) return 64;  // chunks of route_fold_kernel
    if (route_data_uses_mfma(b, l, d, n, bf16)) return 16 * data_mfma_waves(b, l);
    return route_tokens_per_chunk(b, l);
}

constexpr int ROUTE_THREADS = 256;
constexpr int ROUTE_WAVES = ROUTE_THREADS / 64;

template <typename T, int NMAX, bool HAS_E, bool HAS_D>
__global__ __launch_bounds__(ROUTE_THREADS) void route_partial_kernel(RouteArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // Workgroup order: the b samples of one chunk are neighbours in time and sit on the same XCD
    // (workgroup ids are dealt round-robin over the 8 XCDs), so a chunk of W_E is fetched from HBM
    // once and found in that XCD's L2 by the other samples.
    const int lin = blockIdx.x;
    const int chunk = ((lin >> 3) / a.b) * 8 + (lin & 7), bb = (lin >> 3) % a.b;
    if (chunk >= a.nchunks) return;
    const int n = a.n, d = a.d, l = a.l, m = a.m;
    const int t0 = chunk * a.tc;
    const int tcur = min(a.tc, l - t0);

    // LDS carve-up: W_B transposed [n][d] (storage type), t1 [tc][NMAX], zred [waves][NMAX]
    T *wb_t = reinterpret_cast<T *>(smem);
    size_t off = HAS_D ? (((size_t)n * d * sizeof(T) + 15) & ~(size_t)15) : 0;
    float *t1s = reinterpret_cast<float *>(smem + off);
    float *zsh = t1s + (HAS_D ? a.tc * NMAX : 0);

    const T *x = static_cast<const T *>(a.x);
    const T *w_e = static_cast<const T *>(a.w_e);
    if (HAS_D) {
        const T *w_b = static_cast<const T *>(a.w_b);
        for (int idx = tid; idx < n * d; idx += ROUTE_THREADS) {
            const int e = idx / n, i = idx - e * n;  // W_B is [d, n]
            wb_t[i * d + e] = w_b[idx];
        }
        __syncthreads();
    }

    float zacc[NMAX];
#pragma unroll
    for (int i = 0; i < NMAX; ++i) zacc[i] = 0.f;

    // Rows i >= n of the unrolled NMAX loops re-read row n-1 and accumulate into slots that are
    // never written out: the hot loop has no branches, so all NMAX+1 loads of an iteration are in
    // flight together.
    const size_t ld = (size_t)l * d;
    size_t wrow[NMAX];
#pragma unroll
    for (int i = 0; i < NMAX; ++i) wrow[i] = (size_t)min(i, n - 1) * ld;
    for (int tl = wave; tl < tcur; tl += ROUTE_WAVES) {
        const int t = t0 + tl;
        const T *xr = x + ((size_t)bb * l + t) * d;
        float tacc[NMAX];
#pragma unroll
        for (int i = 0; i < NMAX; ++i) tacc[i] = 0.f;
        for (int e = lane * 8; e < d; e += 64 * 8) {
            float xv[8];
            load8(xr + e, xv);
            if (HAS_E) {
                const T *wp = w_e + (size_t)t * d + e;
                float wv[NMAX][8];
#pragma unroll
                for (int i = 0; i < NMAX; ++i) load8(wp + wrow[i], wv[i]);
#pragma unroll
                for (int i = 0; i < NMAX; ++i)
#pragma unroll
                    for (int q = 0; q < 8; ++q) zacc[i] = fmaf(xv[q], wv[i][q], zacc[i]);
            }
            if (HAS_D) {
#pragma unroll
                for (int i = 0; i < NMAX; ++i) {
                    float wv[8];
                    load8(wb_t + min(i, n - 1) * d + e, wv);
#pragma unroll
                    for (int q = 0; q < 8; ++q) tacc[i] = fmaf(xv[q], wv[q], tacc[i]);
                }
            }
        }
        if (HAS_D) {
#pragma unroll
            for (int i = 0; i < NMAX; ++i) {
                const float s = wave_sum(tacc[i]);
                if (lane == 0) t1s[tl * NMAX + i] = s;
            }
        }
    }
    if (HAS_E) {
#pragma unroll
        for (int i = 0; i < NMAX; ++i) {
            const float s = wave_sum(zacc[i]);
            if (lane == 0) zsh[wave * NMAX + i] = s;
        }
    }
    __syncthreads();
    if (HAS_E && tid < n) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < ROUTE_WAVES; ++w) s += zsh[w * NMAX + tid];
        a.zpart[((size_t)chunk * a.b + bb) * n + tid] = s;
    }
    if (HAS_D) {
        const T *w_a = static_cast<const T *>(a.w_a);
        const int nm = n * m;
        for (int o = tid; o < nm; o += ROUTE_THREADS) {
            const int i = o / m, j = o - i * m;
            float s = 0.f;
            for (int tl = 0; tl < tcur; ++tl)
                s = fmaf(t1s[tl * NMAX + i], to_f32(w_a[(size_t)(t0 + tl) * m + j]), s);
            a.gpart[((size_t)chunk * a.b + bb) * nm + o] = s;
        }
    }
}

typedef __bf16 rt_bf16x8 __attribute__((ext_vector_type(8)));
typedef float rt_f32x4 __attribute__((ext_vector_type(4)));

typedef short rt_s16x4 __attribute__((ext_vector_type(4)));
typedef rt_s16x4 __attribute__((address_space(3))) * rt_lds_s16x4_ptr;

// Second half of the data router (Eq. 13): fold per-token expert scores with the chunk's rows of W_A,
// g[i][j] = sum_t t1[t][i] * W_A[t0 + t][j], for the tokens t0 .. t0 + tcur of sample bb, into the
// chunk's partial logit tile gpart[chunk][bb][n*m].  t1s: LDS, [token][np] fp32.  A thread owns
// (token group tg, output group og): one expert i and VEC consecutive patches, for the tokens
// tg, tg + TG, ...; the TG partial sums of an output are then added in group order.  (With few
// outputs per sample, one thread per output would leave most of the workgroup idle behind a
// serial walk over all the chunk's tokens.)  part: LDS scratch of NTHREADS * 8 floats.
// gpart is indexed with the chunk number, W_A with t0 + token unless w_a_rows is given.
template <int NTHREADS>
__device__ __forceinline__ void route_fold(const RouteArgs &a, int chunk, int bb, int t0, int tcur, const float *t1s, int np,
                                           float *part, const uint16_t *w_a_rows = nullptr)
{
    const int tid = threadIdx.x;
    const int n = a.n, m = a.m;
    // rows of W_A: global memory (row t0 + tl), or a copy of the chunk's rows (row tl; the caller passes t0 = 0)
    const uint16_t *w_a = w_a_rows ? w_a_rows : static_cast<const uint16_t *>(a.w_a);
    const int nm = n * m;
    float *gout = a.gpart + ((size_t)chunk * a.b + bb) * nm;
    const int vec = (m & 7) == 0 ? 8 : 1, mv = m / vec, og_n = n * mv;
    const int tg_n = og_n >= NTHREADS ? 1 : NTHREADS / og_n;
    auto fold = [&](int og, int tl0, int tstep, float *dst) {
        const int i = og / mv, j0 = (og - i * mv) * vec;
        float sacc[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) sacc[q] = 0.f;
        if (vec == 8) {
#pragma unroll 4
            for (int tl = tl0; tl < tcur; tl += tstep) {
                float wv[8];
                load8(reinterpret_cast<const bf16_t *>(w_a) + (size_t)(t0 + tl) * m + j0, wv);
                const float t1 = t1s[tl * np + i];
#pragma unroll
                for (int q = 0; q < 8; ++q) sacc[q] = fmaf(t1, wv[q], sacc[q]);
            }
        } else {
#pragma unroll 4
            for (int tl = tl0; tl < tcur; tl += tstep)
                sacc[0] = fmaf(t1s[tl * np + i], __uint_as_float((uint32_t)w_a[(size_t)(t0 + tl) * m + j0] << 16), sacc[0]);
        }
        for (int q = 0; q < vec; ++q) dst[i * m + j0 + q] = sacc[q];
    };
    if (tg_n > 1) {
        const int og = tid % og_n, tg = tid / og_n;
        if (tg < tg_n) fold(og, tg, tg_n, part + (size_t)tg * nm);
        __syncthreads();
        for (int o = tid; o < nm; o += NTHREADS) {
            float t = 0.f;
            for (int q = 0; q < tg_n; ++q) t += part[(size_t)q * nm + o];
            gout[o] = t;
        }
    } else {
        for (int og = tid; og < og_n; og += NTHREADS) fold(og, 0, 1, gout);
    }
}

// W_B [d, n] copied to LDS as it is: rows of NP = 16 or 32 columns (columns >= n are left as they are:
// they only feed output columns that are never read), in blocks of 8 rows with a pad after each block
// (128 bytes for 32-byte rows, 32 bytes for 64-byte rows) so that the row groups of the four k-slices
// of a transposing read fall into different banks.  Row e starts at (e/8)*BLK + (e%8)*ROWB.
template <int NP, int NTHREADS>
__device__ __forceinline__ void stage_w_b(const RouteArgs &a, unsigned char *wb)
{
    constexpr int ROWB = NP * 2, BLK = 8 * ROWB + (NP == 16 ? 128 : 32);
    const int tid = threadIdx.x, n = a.n, d = a.d;
    const uint16_t *w_b = static_cast<const uint16_t *>(a.w_b);
    auto row_at = [&](int e) { return wb + (size_t)(e >> 3) * BLK + (e & 7) * ROWB; };
    if ((n & 7) == 0) {  // 16-byte pieces never straddle a row
        const int pr = n >> 3;
#pragma unroll 4
        for (int idx = tid; idx < d * pr; idx += NTHREADS) {
            const int e = idx / pr, pc = idx - e * pr;
            *reinterpret_cast<uint4 *>(row_at(e) + pc * 16) = *reinterpret_cast<const uint4 *>(w_b + (size_t)idx * 8);
        }
    } else if ((n & 1) == 0) {
        const int pr = n >> 1;
#pragma unroll 4
        for (int idx = tid; idx < d * pr; idx += NTHREADS) {
            const int e = idx / pr, pc = idx - e * pr;
            *reinterpret_cast<uint32_t *>(row_at(e) + pc * 4) = *reinterpret_cast<const uint32_t *>(w_b + (size_t)idx * 2);
        }
    } else {
#pragma unroll 4
        for (int idx = tid; idx < d * n; idx += NTHREADS) {
            const int e = idx / n, i = idx - e * n;
            *reinterpret_cast<uint16_t *>(row_at(e) + i * 2) = w_b[idx];
        }
    }
}

// Data router (Eq. 13), bf16, MFMA.  Workgroup = WAVES waves = WAVES*16 tokens of one sample.
// MFMA 16x16x32 operand layout: lane = (row r = lane%16, k-slice 8*(lane/16)); accumulator register q
// of a lane is output row 4*(lane/16)+q, column lane%16.
// W_B [d, n] is copied to LDS as it is (rows of np = 16 or 32 columns; columns >= n are left as
// they are: they only feed output columns that are never read) and the B fragments (8 consecutive k
// of one expert column) are taken with the transposing LDS read: in a group of 16 lanes, lane j
// points at row k0 + j/4, columns 4*(j%4)..+3, and lane i receives column i, rows k0..k0+3.  Rows are
// stored in blocks of 8 with a pad after each block (128 bytes for 32-byte rows, 32 bytes for
// 64-byte rows) so that the row groups of the four k-slices fall into different banks.
template <int WAVES, int NTILE>
__device__ __forceinline__ void route_data_mfma_body(const RouteArgs &a, int chunk, int bb, unsigned char *smem)
{
    constexpr int NTHREADS = WAVES * 64, TC = WAVES * 16;
    constexpr int NP = NTILE * 16, ROWB = NP * 2, BLK = 8 * ROWB + (NP == 16 ? 128 : 32);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int d = a.d, l = a.l;
    const int np = NP;
    const int t0 = chunk * TC, tcur = min(TC, l - t0);
    unsigned char *wb = smem;                                   // W_B rows, blocked
    float *t1s = reinterpret_cast<float *>(smem + (size_t)((d + 7) / 8) * BLK);  // [TC][np]

    // A fragments of the first steps are requested before the staging copy so both are in flight together
    const int r = lane & 15, ksl = (lane >> 4) * 8;
    const int trow = min(t0 + wave * 16 + r, l - 1);  // rows past the end repeat the last token; never used
    const uint16_t *xr = static_cast<const uint16_t *>(a.x) + ((size_t)bb * l + trow) * d;
    constexpr int UN = 4;  // k-steps whose A fragments are in flight together
    auto load_a = [&](int k0, uint4 (&av)[UN]) {
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int kk = k0 + u * 32 + ksl;
            const bool ok = kk < d;  // slices past d (d % 128 != 0) contribute zero
            av[u] = *reinterpret_cast<const uint4 *>(xr + (ok ? kk : 0));
            if (!ok) av[u] = make_uint4(0, 0, 0, 0);
        }
    };
    uint4 av[UN];
    load_a(0, av);

    auto row_at = [&](int e) { return wb + (size_t)(e >> 3) * BLK + (e & 7) * ROWB; };
    stage_w_b<NP, NTHREADS>(a, wb);
    __syncthreads();

    rt_f32x4 acc[NTILE];  // NTILE tiles of 16 experts
#pragma unroll
    for (int t = 0; t < NTILE; ++t)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[t][q] = 0.f;
    // transposing-read lane roles: k-slice group lane/16, row (lane%16)/4 of the group's 4, 4 columns
    const int tr_row = (lane >> 4) * 8 + ((lane & 15) >> 2), tr_col = (lane & 3) * 4;
    for (int k0 = 0; k0 < d; k0 += 32 * UN) {
        uint4 nv[UN] = {};
        if (k0 + 32 * UN < d) load_a(k0 + 32 * UN, nv);
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            // rows past d: the A side is zero; read a valid row so that the product stays finite
            const int kr = min(k0 + u * 32 + tr_row, d - 8 + ((lane & 15) >> 2));
            const rt_bf16x8 af = __builtin_bit_cast(rt_bf16x8, av[u]);
#pragma unroll
            for (int t = 0; t < NTILE; ++t) {
                const unsigned char *src = row_at(kr) + (t * 16 + tr_col) * 2;
                const rt_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((rt_lds_s16x4_ptr)(src));
                const rt_s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((rt_lds_s16x4_ptr)(row_at(kr + 4) + (t * 16 + tr_col) * 2));
                const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
                const rt_bf16x8 bfr = __builtin_bit_cast(rt_bf16x8, make_uint4(l2.x, l2.y, h2.x, h2.y));
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, bfr, acc[t], 0, 0, 0);
            }
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) av[u] = nv[u];
    }
#pragma unroll
    for (int t = 0; t < NTILE; ++t)
#pragma unroll
        for (int q = 0; q < 4; ++q) t1s[(wave * 16 + (lane >> 4) * 4 + q) * np + t * 16 + r] = acc[t][q];
    __syncthreads();

    route_fold<NTHREADS>(a, chunk, bb, t0, tcur, t1s, np, t1s + TC * np);
}

template <int WAVES, int NTILE>
__global__ __launch_bounds__(WAVES * 64) void route_data_mfma_kernel(RouteArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    route_data_mfma_body<WAVES, NTILE>(a, blockIdx.x, blockIdx.y, smem);
}

// Expert router (Eq. 21), bf16, MFMA.  Workgroup = 4 waves = (chunk of a.tc tokens, i.e. a.tc*d
// consecutive elements of the flat l*d axis; group of RT*16 samples).  The chunk is cut into steps of
// 32 elements; wave w takes a contiguous quarter of the steps.  In one step lane (r = lane%16,
// q = lane/16) loads elements [32*step + 8*q, +8) of sample row r (one A fragment per 16 samples)
// and of expert row r (one B fragment per 16 experts); rows past b or n repeat the last valid row
// (they only produce output rows / columns that are never stored).  The last step of a chunk may
// be partial (multiples of 8 elements): its missing slices are zeroed.  Accumulator register v of
// a lane is Z[sample 4*q + v][expert r].  The four waves' tiles are summed in wave order.
template <int RT, int CT> constexpr size_t route_expert_mfma_lds() { return sizeof(float) * 4 * RT * 16 * (CT * 16 + 1); }

template <int RT, int CT>
__device__ __forceinline__ void route_expert_mfma_body(const RouteArgs &a, int chunk, int b0, unsigned char *smem)
{
    float(*zsh)[RT * 16][CT * 16 + 1] = reinterpret_cast<float(*)[RT * 16][CT * 16 + 1]>(smem);  // [4 waves]
    constexpr int U = 4;  // steps whose loads are in flight together
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, q = lane >> 4;
    const int b = a.b, n = a.n;
    const long ld = (long)a.l * a.d;
    const long c0 = (long)chunk * a.tc * a.d;
    const long c1 = min(ld, c0 + (long)a.tc * a.d);
    const int steps = (int)((c1 - c0 + 31) / 32);
    const int per = (steps + 3) / 4;
    const int s0 = wave * per, s1 = min(steps, s0 + per);

    const uint16_t *xp[RT], *wp[CT];
#pragma unroll
    for (int t = 0; t < RT; ++t) xp[t] = static_cast<const uint16_t *>(a.x) + (size_t)min(b0 + t * 16 + r, b - 1) * ld;
#pragma unroll
    for (int t = 0; t < CT; ++t) wp[t] = static_cast<const uint16_t *>(a.w_e) + (size_t)min(t * 16 + r, n - 1) * ld;
    rt_f32x4 acc[RT][CT];
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int u = 0; u < CT; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[t][u][v] = 0.f;

    // Two register sets: the loads of the next U steps are issued before the MFMAs of the current
    // ones, so a wave always has loads in flight (the kernel is a pure stream: bytes in flight are
    // its throughput).
    uint4 xa[2][U][RT], wb[2][U][CT];
    auto load_steps = [&](int s, int set) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long e = c0 + (long)(s + u) * 32 + q * 8;
            const bool ok = s + u < s1 && e < c1;
            const long ec = ok ? e : c0;  // any valid address
#pragma unroll
            for (int t = 0; t < RT; ++t) {
                xa[set][u][t] = *reinterpret_cast<const uint4 *>(xp[t] + ec);
                if (!ok) xa[set][u][t] = make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int t = 0; t < CT; ++t) wb[set][u][t] = *reinterpret_cast<const uint4 *>(wp[t] + ec);
        }
    };
    auto mfma_steps = [&](int set) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < RT; ++t)
#pragma unroll
                for (int v = 0; v < CT; ++v)
                    acc[t][v] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(rt_bf16x8, xa[set][u][t]),
                                                                        __builtin_bit_cast(rt_bf16x8, wb[set][u][v]), acc[t][v], 0, 0, 0);
    };
    if (s0 < s1) load_steps(s0, 0);
    for (int s = s0; s < s1; s += 2 * U) {
        if (s + U < s1) load_steps(s + U, 1);
        mfma_steps(0);
        if (s + U < s1) {
            if (s + 2 * U < s1) load_steps(s + 2 * U, 0);
            mfma_steps(1);
        }
    }
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int u = 0; u < CT; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v) zsh[wave][t * 16 + q * 4 + v][u * 16 + r] = acc[t][u][v];
    __syncthreads();
    for (int o = tid; o < RT * 16 * CT * 16; o += 256) {
        const int row = o / (CT * 16), col = o - row * (CT * 16);
        if (b0 + row < b && col < n)
            a.zpart[((size_t)chunk * b + b0 + row) * n + col] = (zsh[0][row][col] + zsh[1][row][col]) + (zsh[2][row][col] + zsh[3][row][col]);
    }
}

template <int RT, int CT>
__global__ __launch_bounds__(256) void route_expert_mfma_kernel(RouteArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    route_expert_mfma_body<RT, CT>(a, blockIdx.x, blockIdx.y * RT * 16, smem);
}

// Both routers of a block in one launch (they are independent and both stream x): workgroups
// [0, n_data) run the data router with four waves (chunk = id % nchunks_d, sample = id / nchunks_d) -
// first, because each is a longer chain of dependent steps - and the rest the expert router
// (chunk = id' % nchunks, sample group = id' / nchunks).
template <int RT, int CT>
__global__ __launch_bounds__(256) void route_expert_data_kernel(RouteArgs a, int n_data)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int id = blockIdx.x;
    if (id < n_data) {
        route_data_mfma_body<4, CT>(a, id % a.nchunks_d, id / a.nchunks_d, smem);
    } else {
        const int f = id - n_data;
        route_expert_mfma_body<RT, CT>(a, f % a.nchunks, (f / a.nchunks) * RT * 16, smem);
    }
}

// ---------------------------------------------------------------------------------------------
// Streaming router kernel (bf16, d % 128 == 0): the expert router (Eq. 21) and, optionally, the first
// map of the data router (Eq. 13, t1 = x W_B) in one pass over x.
//
// Eq. 21 is a [b, l*d] x [l*d, n] product with a huge inner dimension and almost no arithmetic: what
// counts is how the bytes are requested.  One workgroup per compute unit owns a contiguous run of
// whole tokens (chunk) for up to RT*16 samples and all experts.  The chunk moves through LDS in
// stages of RB bytes per row (rows = the samples' rows of x, then the experts' rows of W_E), fetched
// by global_load_lds (16 bytes per lane, 1 KiB of consecutive LDS per instruction: whole 0.5-1 KiB
// runs of one row per request, no registers held by loads in flight), three stages deep.  Measured
// against register-staged fragment loads of 64 bytes per row the same stream runs 20 % faster.
// Within a row the 16-byte chunks are permuted (slot = chunk ^ (row & 15), applied on the global
// side where every lane supplies its own address) so that the fragment reads of 16 rows hit 64
// distinct banks.
// MFMA v_mfma_f32_16x16x32_bf16, rows = samples, columns = experts.  A stage holds RB/64 steps of 32
// elements; wave w takes steps w, w+4, ....  For the data router the same x fragment is multiplied a
// second time, with the matching W_B fragment (transposing LDS read of a copy of W_B, as in
// route_data_mfma): since d % 128 == 0 every wave owns d/128 steps of every token, so each wave
// carries one partial row of t1 per token, parks it in LDS when the token ends, and after the stream
// the four partial rows are added in wave order and go to t1 [b][l][n] (fp32) for route_fold_kernel.  Nothing but the stage loads touches vector memory
// inside the loop, whose completion is tracked by hand (s_waitcnt vmcnt) as in the GEMM engine.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void rs_dma16(const void *gptr, uint32_t lds_byte)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_byte), "v"(gptr) : "memory", "m0");
}
// The same with the non-temporal hint, for the rows of W_E: they are read once per call and are larger
// than the memory-side cache, where they would push out x, u and the hidden activations that the
// kernels after the router read again.
__device__ __forceinline__ void rs_dma16_once(const void *gptr, uint32_t lds_byte)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt" ::"s"(lds_byte), "v"(gptr) : "memory", "m0");
}
#pragma clang diagnostic pop
// wait until at most n (0..16) of this wave's vector-memory operations are outstanding
__device__ __forceinline__ void rs_wait(int n)
{
#define UOE_W(N) case N: asm volatile("s_waitcnt vmcnt(" #N ")" ::: "memory"); break;
    switch (n) {
        UOE_W(1) UOE_W(2) UOE_W(3) UOE_W(4) UOE_W(5) UOE_W(6) UOE_W(7) UOE_W(8) UOE_W(9) UOE_W(10) UOE_W(11) UOE_W(12)
        UOE_W(13) UOE_W(14) UOE_W(15) UOE_W(16)
        default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
    }
#undef UOE_W
}

template <int RT, int CT, int RB, bool HAS_D>
__global__ __launch_bounds__(256) void route_stream_kernel(RouteArgs a, int ipw, int once)
{
    constexpr int STAGES = 3, SE = RB / 2, SPS = SE / 32, LPR = RB / 16, RPI = 64 / LPR;
    constexpr int NP = CT * 16, ROWB = NP * 2, BLK = 8 * ROWB + (NP == 16 ? 128 : 32);
    extern __shared__ __align__(1024) unsigned char smem[];
    const int chunk = blockIdx.x, b0 = blockIdx.y * RT * 16;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, q4 = lane >> 4;
    const int b = a.b, n = a.n, d = a.d, l = a.l;
    const long ld = (long)l * d;
    const int bg = min(RT * 16, b - b0), rows = bg + n;
    const int t0 = chunk * a.tc, tcur = min(a.tc, l - t0);
    const long c0 = (long)t0 * d;
    const int spt = d / 32;                       // steps per token
    const int gsteps = tcur * spt;                // steps of this chunk
    const int nst = (gsteps + SPS - 1) / SPS;
    const int SB = ipw * 4 * 1024;                // bytes of one stage buffer

    unsigned char *stage0 = smem;
    float(*zsh)[RT * 16][NP + 1] = reinterpret_cast<float(*)[RT * 16][NP + 1]>(smem + (size_t)STAGES * SB);
    unsigned char *wb = reinterpret_cast<unsigned char *>(&zsh[4][0][0]);
    float *t1w = reinterpret_cast<float *>(wb + (size_t)(d / 8) * BLK);   // [4 waves][tc][bg][n]
    auto row_at = [&](int e) { return wb + (size_t)(e >> 3) * BLK + (e & 7) * ROWB; };
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;

    // stage st -> buffer buf: instruction I = wave + 4 i fills LDS rows I*RPI .. of the stage
    auto issue = [&](int st, int buf) {
        for (int i = 0; i < ipw; ++i) {
            const int ins = wave + 4 * i;
            const int row = ins * RPI + lane / LPR, rc = min(row, rows - 1);
            const uint16_t *base = rc < bg ? static_cast<const uint16_t *>(a.x) + (size_t)(b0 + rc) * ld
                                           : static_cast<const uint16_t *>(a.w_e) + (size_t)(rc - bg) * ld;
            long e = c0 + (long)st * SE + (((lane % LPR) ^ (row & 15)) * 8);
            e = e < ld - 8 ? e : ld - 8;           // past the end of the row: any valid address (never used)
            if (once && ins * RPI >= bg) rs_dma16_once(base + e, lds_base + buf * SB + ins * 1024);   // all rows of the instruction are W_E's (wave-uniform)
            else rs_dma16(base + e, lds_base + buf * SB + ins * 1024);
        }
    };
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s)
        if (s < nst) issue(s, s);
    if (HAS_D) stage_w_b<NP, 256>(a, wb);

    rt_f32x4 accz[RT][CT], acct[RT][CT];
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int u = 0; u < CT; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v) accz[t][u][v] = acct[t][u][v] = 0.f;
    int xoff[RT], woff[CT];   // byte offsets of this lane's fragment rows inside a stage, chunk XOR term separate
    int xsw[RT], wsw[CT];
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        const int row = min(t * 16 + r, bg - 1);
        xoff[t] = row * RB;
        xsw[t] = row & 15;
    }
#pragma unroll
    for (int t = 0; t < CT; ++t) {
        const int row = bg + min(t * 16 + r, n - 1);
        woff[t] = row * RB;
        wsw[t] = row & 15;
    }
    const int tr_row = q4 * 8 + ((lane & 15) >> 2), tr_col = (lane & 3) * 4;

    int tk = 0, sq = wave;   // token and step-in-token of this wave's next step (its steps are wave, wave + 4, ...)
    int buf = 0, nbuf = STAGES - 1;
    for (int st = 0; st < nst; ++st) {
        if (st + STAGES - 1 < nst) rs_wait(ipw); else rs_wait(0);
        __syncthreads();   // stage st has landed for every wave; the buffer of stage st-1 is free
        if (st + STAGES - 1 < nst) issue(st + STAGES - 1, nbuf);
        const unsigned char *sb = stage0 + (size_t)buf * SB;
        // steps wave, wave + 4, ... of the stage: the x fragment feeds both products
#pragma unroll
        for (int u = 0; u < SPS / 4; ++u) {
            const int sl = u * 4 + wave;
            if (st * SPS + sl < gsteps) {
                const int c = sl * 4 + q4;
                rt_bf16x8 wf[CT], bfr[CT], xf[RT];
#pragma unroll
                for (int v = 0; v < CT; ++v) wf[v] = *reinterpret_cast<const rt_bf16x8 *>(sb + woff[v] + ((c ^ wsw[v]) * 16));
#pragma unroll
                for (int t = 0; t < RT; ++t) xf[t] = *reinterpret_cast<const rt_bf16x8 *>(sb + xoff[t] + ((c ^ xsw[t]) * 16));
                if (HAS_D) {
                    const int kr = sq * 32 + tr_row;   // W_B row = feature index of the step
#pragma unroll
                    for (int v = 0; v < CT; ++v) {
                        const rt_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((rt_lds_s16x4_ptr)(row_at(kr) + (v * 16 + tr_col) * 2));
                        const rt_s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((rt_lds_s16x4_ptr)(row_at(kr + 4) + (v * 16 + tr_col) * 2));
                        const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
                        bfr[v] = __builtin_bit_cast(rt_bf16x8, make_uint4(l2.x, l2.y, h2.x, h2.y));
                    }
                }
#pragma unroll
                for (int t = 0; t < RT; ++t)
#pragma unroll
                    for (int v = 0; v < CT; ++v) {
                        accz[t][v] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[t], wf[v], accz[t][v], 0, 0, 0);
                        if (HAS_D) acct[t][v] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[t], bfr[v], acct[t][v], 0, 0, 0);
                    }
                if (HAS_D) {
                    sq += 4;
                    if (sq >= spt) {   // this wave's share of token tk is complete
#pragma unroll
                        for (int t = 0; t < RT; ++t)
#pragma unroll
                            for (int v = 0; v < CT; ++v)
#pragma unroll
                                for (int w = 0; w < 4; ++w) {
                                    const int row = t * 16 + q4 * 4 + w, col = v * 16 + r;
                                    if (row < bg && col < n) t1w[(((size_t)wave * a.tc + tk) * bg + row) * n + col] = acct[t][v][w];
                                    acct[t][v][w] = 0.f;
                                }
                        sq -= spt;
                        ++tk;
                    }
                }
            }
        }
        buf = buf + 1 == STAGES ? 0 : buf + 1;
        nbuf = nbuf + 1 == STAGES ? 0 : nbuf + 1;
    }
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int u = 0; u < CT; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v) zsh[wave][t * 16 + q4 * 4 + v][u * 16 + r] = accz[t][u][v];
    __syncthreads();
    for (int o = tid; o < RT * 16 * NP; o += 256) {
        const int row = o / NP, col = o - row * NP;
        if (row < bg && col < n)
            a.zpart[((size_t)chunk * b + b0 + row) * n + col] = (zsh[0][row][col] + zsh[1][row][col]) + (zsh[2][row][col] + zsh[3][row][col]);
    }
    if (HAS_D) {
        for (int o = tid; o < tcur * bg * n; o += 256) {
            const int i = o % n, bb = (o / n) % bg, tl = o / (n * bg);
            const size_t at = ((size_t)tl * bg + bb) * n + i, ws = (size_t)a.tc * bg * n;
            a.t1[((size_t)(b0 + bb) * l + t0 + tl) * n + i] = (t1w[at] + t1w[ws + at]) + (t1w[2 * ws + at] + t1w[3 * ws + at]);
        }
    }
}

// Second kernel of the one-pass routing: workgroup = (chunk of a.tc_d tokens, sample).  The chunk's
// rows of t1 and of W_A go to LDS with every load of the workgroup in flight at once (the fold
// itself is a short loop per thread; fed from global memory it is a chain of load latencies), then
// the fold writes the chunk's partial logit tile (summed by route_reduce or route_select, exactly
// as the partial tiles of route_data_mfma are).
__global__ __launch_bounds__(256) void route_fold_kernel(RouteArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int chunk = blockIdx.x, bb = blockIdx.y, n = a.n, m = a.m;
    const int t0 = chunk * a.tc_d, tcur = min(a.tc_d, a.l - t0);
    uint16_t *wa_s = reinterpret_cast<uint16_t *>(smem);                                            // [tc_d][m]
    float *t1s = reinterpret_cast<float *>(smem + (((size_t)a.tc_d * m * 2 + 15) & ~(size_t)15));   // [tc_d][n]
    const uint16_t *wa_g = static_cast<const uint16_t *>(a.w_a) + (size_t)t0 * m;
    const int wa_elems = tcur * m;
    if ((m & 7) == 0) {
        for (int o = threadIdx.x * 8; o < wa_elems; o += 256 * 8)
            *reinterpret_cast<uint4 *>(wa_s + o) = *reinterpret_cast<const uint4 *>(wa_g + o);
    } else {
        for (int o = threadIdx.x; o < wa_elems; o += 256) wa_s[o] = wa_g[o];
    }
    const float *src = a.t1 + ((size_t)bb * a.l + t0) * n;
    for (int o = threadIdx.x; o < tcur * n; o += 256) t1s[o] = src[o];
    __syncthreads();
    route_fold<256>(a, chunk, bb, 0, tcur, t1s, n, t1s + (size_t)a.tc_d * n, wa_s);
}

// The fold of the one-pass routing on the matrix cores (n*m outputs per sample, l products each: 67 M
// multiply-adds on the largest shape, a latency chain on the vector ALU).  Workgroup = (token range,
// sample); g[i][j] += sum_t t1[t][i] * W_A[t][j] as v_mfma_f32_16x16x32_bf16 with rows = experts,
// columns = patches, k = 32 tokens.  t1 is fp32 and selection has to agree with an fp64 reference to
// 1e-5 relative, so it enters as three bf16 terms, t1 = hi + mid + lo (each the rounded remainder of
// the ones before: 24 significant bits, exact to fp32), three MFMAs against the same W_A fragment.
// Wave w takes the 32-token steps w, w+4, ... of the range (at most 4): A fragments straight from global memory
// (lane (i, q) holds tokens 8q..8q+7 of expert i), the step's rows of W_A through a wave-private LDS
// tile and the transposing LDS read.  The four waves' tiles are added in wave order.
constexpr int FOLD_MAX_M = 128;   // accumulators: (m/16) x (n/16) tiles of 4 registers; LDS within 64 KiB
static bool route_fold_mfma_ok(int n, int m)
{
    if ((m & 7) != 0 && m > 16) return false;   // the W_A rows of a step: at most 8 loads per lane
    return n <= 16 ? m <= FOLD_MAX_M : m <= FOLD_MAX_M / 2;
}
// MT = column tiles computed (>= ceil(m/16); tiles past m work on zero-filled LDS columns and are not stored),
// STEPS = 32-token steps per wave (steps past the range work on zeros): straight-line code, no
// accumulator ever crosses a branch.
template <int CT, int MT, int STEPS>
__global__ __launch_bounds__(256) void route_fold_mfma_kernel(RouteArgs a, int tr)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i16 = lane & 15, q4 = lane >> 4;
    const int n = a.n, m = a.m, l = a.l, nm = n * m;
    const int rg = blockIdx.x, bb = blockIdx.y;
    const int t_begin = rg * tr, t_end = min(l, t_begin + tr);
    constexpr int pitch = 2 * b_pitch16(MT * 16);                  // elements per LDS row of W_A
    uint16_t *wa_s = reinterpret_cast<uint16_t *>(smem) + (size_t)wave * 32 * pitch;   // [32 tokens][pitch], this wave's
    float *red = reinterpret_cast<float *>(smem);   // [4 waves][CT*16][MT*16], over the W_A tiles once every wave is done with them

    rt_f32x4 acc[CT][MT];
#pragma unroll
    for (int c = 0; c < CT; ++c)
#pragma unroll
        for (int j = 0; j < MT; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[c][j][v] = 0.f;
    const float *t1 = a.t1 + (size_t)bb * l * n;
    const uint16_t *w_a = static_cast<const uint16_t *>(a.w_a);
    const int tr_row = q4 * 8 + ((lane & 15) >> 2), tr_col = (lane & 3) * 4;

    // A dependent memory round trip costs microseconds here, so ALL loads of the wave (8 values of t1 and
    // PC pieces of W_A per lane and step, none depending on another) are issued before anything else.
    // W_A rows: 16-byte pieces when m % 8 == 0 (a row of the LDS tile = MT*2 pieces, columns past m come
    // from the next row and are never used), single elements otherwise (m <= 16).
    const bool vec = (m & 7) == 0;
    // pieces per lane and step: 32 rows * (m/8 <= 2 MT) / 64 lanes; up to 32 * 16 / 64 single elements when m <= 16
    constexpr int PC = MT == 1 ? 8 : (MT <= 4 ? MT : 8);
    const int pr = vec ? m >> 3 : m;                // pieces per row
    int prow[PC], goff[PC], loff[PC];
#pragma unroll
    for (int u = 0; u < PC; ++u) {
        const int idx = lane + 64 * u, row = idx / pr, within = idx - row * pr;
        prow[u] = row;                              // rows >= 32 are never loaded or stored
        goff[u] = vec ? row * m + within * 8 : idx;
        loff[u] = row * pitch + (vec ? within * 8 : within);
    }
    float tv[STEPS][CT][8];
    uint4 wv[STEPS][PC];
    uint16_t we[STEPS][PC];
#pragma unroll
    for (int sidx = 0; sidx < STEPS; ++sidx) {
        const int k0 = t_begin + (wave + 4 * sidx) * 32;
#pragma unroll
        for (int c = 0; c < CT; ++c)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int t = k0 + q4 * 8 + e, i = c * 16 + i16;
                const bool ok = t < t_end && i < n;       // tokens past the range contribute zero
                tv[sidx][c][e] = t1[ok ? (size_t)t * n + i : (size_t)t_begin * n];
                if (!ok) tv[sidx][c][e] = 0.f;
            }
#pragma unroll
        for (int u = 0; u < PC; ++u) {
            const bool ok = prow[u] < 32 && k0 + prow[u] < t_end;
            const size_t at = ok ? (size_t)k0 * m + goff[u] : (size_t)0;
            if (vec) {
                wv[sidx][u] = *reinterpret_cast<const uint4 *>(w_a + (at & ~(size_t)7));
                if (!ok) wv[sidx][u] = make_uint4(0, 0, 0, 0);
            } else {
                we[sidx][u] = w_a[at];
                if (!ok) we[sidx][u] = 0;
            }
        }
    }
#pragma unroll
    for (int sidx = 0; sidx < STEPS; ++sidx) {
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < PC; ++u) {
            if (prow[u] < 32) {
                if (vec) *reinterpret_cast<uint4 *>(wa_s + loff[u]) = wv[sidx][u];
                else wa_s[loff[u]] = we[sidx][u];
            }
        }
        __builtin_amdgcn_wave_barrier();   // a wave reads back only what it wrote itself; LDS runs one wave's instructions in order
        rt_bf16x8 af[CT][3];
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            uint32_t w3[3][4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float r0 = tv[sidx][c][2 * e], r1 = tv[sidx][c][2 * e + 1];
#pragma unroll
                for (int term = 0; term < 3; ++term) {
                    const uint32_t h0 = f32_to_bf16_bits(r0), h1 = f32_to_bf16_bits(r1);
                    w3[term][e] = h0 | (h1 << 16);
                    r0 -= __uint_as_float(h0 << 16);
                    r1 -= __uint_as_float(h1 << 16);
                }
            }
#pragma unroll
            for (int term = 0; term < 3; ++term)
                af[c][term] = __builtin_bit_cast(rt_bf16x8, make_uint4(w3[term][0], w3[term][1], w3[term][2], w3[term][3]));
        }
#pragma unroll
        for (int j = 0; j < MT; ++j) {
            const uint16_t *src = wa_s + tr_row * pitch + j * 16 + tr_col;
            const rt_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((rt_lds_s16x4_ptr)(src));
            const rt_s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((rt_lds_s16x4_ptr)(src + 4 * pitch));
            const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
            const rt_bf16x8 bfr = __builtin_bit_cast(rt_bf16x8, make_uint4(l2.x, l2.y, h2.x, h2.y));
#pragma unroll
            for (int c = 0; c < CT; ++c)
#pragma unroll
                for (int term = 2; term >= 0; --term)   // small terms first
                    acc[c][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[c][term], bfr, acc[c][j], 0, 0, 0);
        }
    }
    // accumulator register v of lane (i16, q4) in tile (c, j) is expert c*16 + 4*q4 + v, patch j*16 + i16
    constexpr int mp = MT * 16;
    __syncthreads();
#pragma unroll
    for (int c = 0; c < CT; ++c)
#pragma unroll
        for (int j = 0; j < MT; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) red[((size_t)wave * CT * 16 + c * 16 + q4 * 4 + v) * mp + j * 16 + i16] = acc[c][j][v];
    __syncthreads();
    float *gout = a.gpart + ((size_t)rg * a.b + bb) * nm;
    constexpr size_t ws = (size_t)CT * 16 * mp;
    for (int o = tid; o < nm; o += 256) {
        const int i = o / m, j = o - i * m;
        const size_t at = (size_t)i * mp + j;
        gout[o] = (red[at] + red[ws + at]) + (red[2 * ws + at] + red[3 * ws + at]);
    }
}

// Sums the data router's per-chunk partials in a fixed order (deterministic).  A block owns 16
// reduced values of one sample; thread (value, chunk group) adds every 16th chunk, then the 16
// group sums are added in group order.  (The expert router's n values per sample are summed by
// route_select itself.)
__global__ __launch_bounds__(256) void route_reduce_kernel(RouteArgs a)
{
    __shared__ float part[16][17];
    const int bb = blockIdx.y, vi = threadIdx.x & 15, cg = threadIdx.x >> 4;
    const int nm = a.n * a.m;
    const int v = blockIdx.x * 16 + vi;
    float s = 0.f;
    if (v < nm) {
        const float *src = a.gpart + (size_t)bb * nm + v;
        const size_t stride = (size_t)a.b * nm;
        for (int ch = cg; ch < a.nchunks_d; ch += 16) s += src[(size_t)ch * stride];
    }
    part[cg][vi] = s;
    __syncthreads();
    if (threadIdx.x < 16 && v < nm) {
        float t = 0.f;
#pragma unroll
        for (int q = 0; q < 16; ++q) t += part[q][vi];
        a.gred[(size_t)bb * nm + v] = t;
    }
}

// One workgroup per (expert i, sample): top-c of row i of the patch gate; the workgroup of expert 0
// also does the sample's top-k over experts.  LDS: ranking keys of the row [m] + kept flags [m]
// (+ the sample's n*m noisy logits when they fit: `staged`).  The kernel is a chain of small
// dependent steps, so everything it needs from global memory is fetched up front by loops whose
// loads do not depend on each other (unrolled: several in flight), never inside the chains.
constexpr int SELECT_THREADS = 512;
constexpr size_t SELECT_STAGE_MAX = 32 * 1024;  // bytes of logits staged in LDS
// fuse_reduce: the data router's per-chunk partials are summed here (each of the n workgroups of
// a sample repeats the sum: worth it only while n*m*chunks is small) instead of by route_reduce.
__global__ __launch_bounds__(SELECT_THREADS) void route_select_kernel(RouteArgs a, int has_e, int has_d, int staged,
                                                                      int fuse_reduce)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, i = blockIdx.x, bb = blockIdx.y;
    const int n = a.n, m = a.m, c = a.c, k = a.k, nm = n * m;
    float *key = reinterpret_cast<float *>(smem);
    unsigned char *kept = smem + (size_t)m * sizeof(float);
    float *glog = reinterpret_cast<float *>(smem + (((size_t)m * 5 + 15) & ~(size_t)15));  // [n*m] when staged
    __shared__ float ge[32];
    __shared__ float zpart_sum[SELECT_THREADS];
    __shared__ float dpart[SELECT_THREADS];
    __shared__ unsigned char ekept[32];
    const float *gsrc = a.gred + (size_t)bb * nm;

    // the expert router's per-chunk partials, summed in a fixed order: thread = (chunk group, expert)
    const int groups = SELECT_THREADS / n;  // >= 16
    float zs = 0.f;
    if (has_e && i == 0 && tid < groups * n) {
        const int vi = tid % n, cg = tid / n;
        const float *src = a.zpart + (size_t)bb * n + vi;
        const size_t stride = (size_t)a.b * n;
#pragma unroll 8
        for (int ch = cg; ch < a.nchunks; ch += groups) zs += src[(size_t)ch * stride];
    }
    if (has_d && staged) {
        const float *nzs = a.noise_p ? a.noise_p + (size_t)bb * nm : nullptr;
        if (fuse_reduce == 2) {  // few partial tiles of any size: every thread adds up its values in tile order
            const float *src = a.gpart + (size_t)bb * nm;
            const size_t stride = (size_t)a.b * nm;
            // four values per thread and pass, at most 16 tiles each (route_fold_plan): all loads of a pass in
            // flight together, tiles added in order
            for (int base = 0; base < nm; base += 4 * SELECT_THREADS) {
                float pv[4][16];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int idx = base + q * SELECT_THREADS + tid;
#pragma unroll
                    for (int ch = 0; ch < 16; ++ch) pv[q][ch] = (idx < nm && ch < a.nchunks_d) ? src[(size_t)ch * stride + idx] : 0.f;
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int idx = base + q * SELECT_THREADS + tid;
                    if (idx < nm) {
                        float t = nzs ? nzs[idx] : 0.f;
#pragma unroll
                        for (int ch = 0; ch < 16; ++ch) t += pv[q][ch];
                        glog[idx] = t;
                    }
                }
            }
        } else if (fuse_reduce) {  // nm <= SELECT_THREADS: thread = (chunk group, value), groups summed in order
            const float *src = a.gpart + (size_t)bb * nm;
            const size_t stride = (size_t)a.b * nm;
            const int dgroups = SELECT_THREADS / nm, v = tid % nm, cg = tid / nm;
            float s = 0.f;
            if (cg < dgroups) {
#pragma unroll 8
                for (int ch = cg; ch < a.nchunks_d; ch += dgroups) s += src[(size_t)ch * stride + v];
                dpart[tid] = s;
            }
            __syncthreads();
            if (tid < nm) {
                float t = nzs ? nzs[tid] : 0.f;
                for (int q = 0; q < dgroups; ++q) t += dpart[q * nm + tid];
                glog[tid] = t;
            }
        } else {
#pragma unroll 8
            for (int idx = tid; idx < nm; idx += SELECT_THREADS) glog[idx] = gsrc[idx] + (nzs ? nzs[idx] : 0.f);
        }
        __syncthreads();
    }

    // ---- data selection: Eq. 13 logits (+noise) -> Eq. 14 gate -> Eq. 17 top-c of row i
    for (int j = tid; j < m; j += SELECT_THREADS) {
        float kv = 0.f, gate = 1.f;
        if (has_d && staged) {  // softmax over the n experts of patch j, logits from LDS
            float mx = -INFINITY;
            for (int ii = 0; ii < n; ++ii) mx = fmaxf(mx, glog[ii * m + j]);
            float den = 0.f;
            for (int ii = 0; ii < n; ++ii) den += expf(glog[ii * m + j] - mx);
            const float own = glog[i * m + j];
            gate = expf(own - mx) / den;
            kv = (own - mx) - logf(den);  // ranking key: see below
        } else if (has_d) {  // the same straight from global memory
            const float *col = gsrc + j;
            const float *nz = a.noise_p ? a.noise_p + (size_t)bb * nm + j : nullptr;
            float mx = -INFINITY, own = 0.f;
            for (int ii = 0; ii < n; ++ii) {
                const float v = col[(size_t)ii * m] + (nz ? nz[(size_t)ii * m] : 0.f);
                mx = fmaxf(mx, v);
                if (ii == i) own = v;
            }
            float den = 0.f;
            for (int ii = 0; ii < n; ++ii) den += expf(col[(size_t)ii * m] + (nz ? nz[(size_t)ii * m] : 0.f) - mx);
            gate = expf(own - mx) / den;
            // ranking key: the log of the gate.  Same order as the gate itself, but a gate too
            // small for fp32 keeps its rank instead of collapsing into a tie at zero.
            kv = (own - mx) - logf(den);
        }
        key[j] = kv;
        if (a.patch_gate) a.patch_gate[(size_t)bb * nm + (size_t)i * m + j] = gate;
    }
    __syncthreads();
    for (int j = tid; j < m; j += SELECT_THREADS) {
        const float v = key[j];
        int rank = 0;
        for (int jj = 0; jj < m; ++jj) {
            const float w = key[jj];
            rank += (w > v || (w == v && jj < j)) ? 1 : 0;
        }
        kept[j] = rank < c;
    }
    __syncthreads();
    if (a.patch_idx) {
        for (int j = tid; j < m; j += SELECT_THREADS) {
            if (!kept[j]) continue;
            int pos = 0;
            for (int jj = 0; jj < j; ++jj) pos += kept[jj];
            a.patch_idx[((size_t)bb * n + i) * c + pos] = j;
        }
    }
    if (i != 0) return;  // uniform per workgroup

    // ---- dynamic capacity (Eq. 15-16) and balance statistics (Eq. 43-44), from the staged logits.
    // Stage 1: patch j names its patch_k best experts (rank counting on the logits, which order the
    // experts of one patch exactly as the gates do; ties to the lower index); count_i = number of
    // patches that named expert i (integer LDS adds: order-independent); c = max_i count_i.
    if (a.capacity && has_d && staged) {  // uniform
        __shared__ int ccount[32];
        if (tid < n) ccount[tid] = 0;
        __syncthreads();  // also: every thread is past its last read of glog as logits of row 0
        for (int j = tid; j < m; j += SELECT_THREADS) {
            float mx = -INFINITY;
            for (int ii = 0; ii < n; ++ii) mx = fmaxf(mx, glog[ii * m + j]);
            float den = 0.f;
            for (int ii = 0; ii < n; ++ii) den += expf(glog[ii * m + j] - mx);
            for (int ii = 0; ii < n; ++ii) {
                const float v = glog[ii * m + j];
                int rank = 0;
                for (int t = 0; t < n; ++t) {
                    const float w = glog[t * m + j];
                    rank += (w > v || (w == v && t < ii)) ? 1 : 0;
                }
                if (rank < a.patch_k) atomicAdd(&ccount[ii], 1);
            }
            // this thread alone owns column j: the logits can now be replaced by the gates
            for (int ii = 0; ii < n; ++ii) glog[ii * m + j] = expf(glog[ii * m + j] - mx) / den;
        }
        __syncthreads();
        if (tid < n) {
            if (a.load_f) a.load_f[(size_t)bb * n + tid] = (float)n * (float)ccount[tid] / ((float)a.patch_k * (float)m);
            if (a.load_p) {
                float sum = 0.f;
                for (int j = 0; j < m; ++j) sum += glog[tid * m + j];  // fixed order
                a.load_p[(size_t)bb * n + tid] = sum / (float)m;
            }
        }
        if (tid == 0) {
            int cmax = 0;
            for (int ii = 0; ii < n; ++ii) cmax = max(cmax, ccount[ii]);
            a.capacity[bb] = cmax;
        }
    }

    // ---- expert selection: Eq. 21 logits (+noise) -> softmax -> Eq. 22 top-k
    // The softmax is strictly increasing in the logit within a sample, so the k largest gates are
    // the k largest logits: rank on the logits, which cannot underflow.
    if (has_e && tid < groups * n) zpart_sum[tid] = zs;  // index = group * n + expert
    __syncthreads();
    float z = 0.f;
    if (tid < n) {
        if (has_e) {
            for (int cg = 0; cg < groups; ++cg) z += zpart_sum[cg * n + tid];
            if (a.noise_e) z += a.noise_e[(size_t)bb * n + tid];
        }
        ge[tid] = z;
    }
    __syncthreads();
    if (tid < n) {
        float gv = 1.0f;
        if (has_e) {
            float mx = -INFINITY;
            for (int ii = 0; ii < n; ++ii) mx = fmaxf(mx, ge[ii]);
            float den = 0.f;
            for (int ii = 0; ii < n; ++ii) den += expf(ge[ii] - mx);
            gv = expf(z - mx) / den;
        }
        if (a.expert_gate) a.expert_gate[(size_t)bb * n + tid] = gv;
        int rank = 0;
        for (int ii = 0; ii < n; ++ii) rank += (ge[ii] > z || (ge[ii] == z && ii < tid)) ? 1 : 0;
        ekept[tid] = rank < k;
    }
    __syncthreads();
    if (tid < n && ekept[tid] && a.expert_idx) {
        int pos = 0;
        for (int ii = 0; ii < tid; ++ii) pos += ekept[ii];
        a.expert_idx[(size_t)bb * k + pos] = tid;
    }
}

// Eq. 42 per sample and its gradient through P_i = mean_j g_{i,j} (Eq. 44); f_i (Eq. 43) is a count.
// One workgroup per sample; the n products are added in expert order.
__global__ __launch_bounds__(256) void balance_loss_kernel(const float *load_f, const float *load_p, float alpha, float *loss,
                                                           float *d_patch_gate, int n, int m)
{
    const int bb = blockIdx.x, tid = threadIdx.x;
    const float *f = load_f + (size_t)bb * n;
    if (loss && tid == 0) {
        const float *pr = load_p + (size_t)bb * n;
        float s = 0.f;
        for (int i = 0; i < n; ++i) s += f[i] * pr[i];
        loss[bb] = alpha * s;
    }
    if (d_patch_gate) {
        float *dg = d_patch_gate + (size_t)bb * n * m;
        const float scale = alpha / (float)m;
        for (int idx = tid; idx < n * m; idx += 256) dg[idx] += scale * f[idx / m];
    }
}

hipError_t launch_balance_loss(const float *load_f, const float *load_p, float alpha, float *loss, float *d_patch_gate,
                               int b, int n, int m, hipStream_t st)
{
    hipLaunchKernelGGL(balance_loss_kernel, dim3(b), dim3(256), 0, st, load_f, load_p, alpha, loss, d_patch_gate, n, m);
    return hipGetLastError();
}

template <typename T, int NMAX>
static hipError_t launch_partial(const RouteArgs &a, bool has_e, bool has_d, hipStream_t st)
{
    dim3 grid(((a.nchunks + 7) / 8) * 8 * a.b), block(ROUTE_THREADS);
    size_t sh = 0;
    if (has_d) sh += (((size_t)a.n * a.d * sizeof(T) + 15) & ~(size_t)15) + (size_t)a.tc * NMAX * sizeof(float);
    sh += (size_t)ROUTE_WAVES * NMAX * sizeof(float);
    if (has_e && has_d)
        hipLaunchKernelGGL((route_partial_kernel<T, NMAX, true, true>), grid, block, sh, st, a);
    else if (has_e)
        hipLaunchKernelGGL((route_partial_kernel<T, NMAX, true, false>), grid, block, sh, st, a);
    else
        hipLaunchKernelGGL((route_partial_kernel<T, NMAX, false, true>), grid, block, sh, st, a);
    return hipGetLastError();
}

template <typename T>
static hipError_t launch_partial_n(const RouteArgs &a, bool has_e, bool has_d, hipStream_t st)
{
    if (a.n <= 2) return launch_partial<T, 2>(a, has_e, has_d, st);
    if (a.n <= 4) return launch_partial<T, 4>(a, has_e, has_d, st);
    if (a.n <= 6) return launch_partial<T, 6>(a, has_e, has_d, st);
    if (a.n <= 8) return launch_partial<T, 8>(a, has_e, has_d, st);
    if (a.n <= 12) return launch_partial<T, 12>(a, has_e, has_d, st);
    if (a.n <= 16) return launch_partial<T, 16>(a, has_e, has_d, st);
    if (a.n <= 24) return launch_partial<T, 24>(a, has_e, has_d, st);
    return launch_partial<T, 32>(a, has_e, has_d, st);
}

// dynamic LDS above 64 KiB has to be allowed per kernel (once per device is enough)
template <int RT, int CT, int RB, bool HAS_D>
static hipError_t launch_stream(const RouteArgs &a, const RouteStreamPlan &sp, dim3 grid, hipStream_t st)
{
    static bool allowed[64] = {};
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    if (dev >= 0 && dev < 64 && !allowed[dev]) {
        err = hipFuncSetAttribute(reinterpret_cast<const void *>(&route_stream_kernel<RT, CT, RB, HAS_D>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (err != hipSuccess) return err;
        allowed[dev] = true;
    }
    // W_E is read once per call: non-temporal from the size on that stream_once names (always, at the sizes this kernel is chosen for)
    const int once = stream_once((size_t)a.n * a.l * a.d * 2) ? 1 : 0;
    hipLaunchKernelGGL((route_stream_kernel<RT, CT, RB, HAS_D>), grid, dim3(256), sp.lds, st, a, sp.ipw, once);
    return hipGetLastError();
}

hipError_t launch_route(const RouteArgs &a_in, bool bf16, hipStream_t st)
{
    RouteArgs a = a_in;
    const bool has_e = a.w_e != nullptr, has_d = a.w_b != nullptr;
    hipError_t err = hipSuccess;
    const bool data_mfma = has_d && route_data_uses_mfma(a.b, a.l, a.d, a.n, bf16);
    const int rt = a.b > 32 ? 4 : (a.b > 16 ? 2 : 1);
    const int groups_e = (a.b + rt * 16 - 1) / (rt * 16);
    int fold_ranges = 0;   // > 0: partial tiles of route_fold_mfma, few enough for route_select to add up
    const RouteStreamPlan sp = route_stream_plan(a.b, a.l, a.d, a.n, bf16, has_d);
    if (has_e && sp.ok && route_stream_pays(a.b, a.l, a.d, a.n)) {
        // streaming kernel: expert router and the data router's first map in one pass over x, then the fold
        a.tc = sp.tpc;
        a.nchunks = sp.nchunks;
        const dim3 grid(sp.nchunks, (a.b + sp.rt * 16 - 1) / (sp.rt * 16));
#define UOE_STREAM(RT, CT, RB)                                                                                              \
    do {                                                                                                                    \
        if (has_d) err = launch_stream<RT, CT, RB, true>(a, sp, grid, st);                                                   \
        else err = launch_stream<RT, CT, RB, false>(a, sp, grid, st);                                                        \
    } while (0)
        if (sp.ct == 1) {
            if (sp.rt == 4) UOE_STREAM(4, 1, 512);
            else if (sp.rt == 2) UOE_STREAM(2, 1, 512);
            else UOE_STREAM(1, 1, 1024);
        } else {
            if (sp.rt == 4) UOE_STREAM(4, 2, 512);
            else if (sp.rt == 2) UOE_STREAM(2, 2, 512);
            else UOE_STREAM(1, 2, 1024);
        }
#undef UOE_STREAM
        if (err != hipSuccess) return err;
        if (has_d && route_fold_mfma_ok(a.n, a.m)) {
            // fold on the matrix cores: a few token ranges per sample, summed by route_select itself
            const RouteFoldPlan fp = route_fold_plan(a.b, a.l);
            a.tc_d = fp.tr;
            a.nchunks_d = fp.ranges;
            const int mt = (a.m + 15) / 16, ct = a.n <= 16 ? 1 : 2;
            const int mtt = mt <= 1 ? 1 : (mt <= 2 ? 2 : (mt <= 4 ? 4 : 8)), steps = fp.tr <= 128 ? 1 : (fp.tr <= 256 ? 2 : 4);
            const size_t sh_wa = (size_t)4 * 32 * 2 * b_pitch16(mtt * 16) * 2, sh_red = (size_t)4 * ct * 16 * mtt * 16 * sizeof(float);
            const size_t shf = sh_wa > sh_red ? sh_wa : sh_red;
            const dim3 grid(fp.ranges, a.b);
#define UOE_FOLD3(CT, MT, ST) hipLaunchKernelGGL((route_fold_mfma_kernel<CT, MT, ST>), grid, dim3(256), shf, st, a, fp.tr)
#define UOE_FOLD2(CT, MT) do { if (steps == 1) UOE_FOLD3(CT, MT, 1); else if (steps == 2) UOE_FOLD3(CT, MT, 2); else UOE_FOLD3(CT, MT, 4); } while (0)
#define UOE_FOLD1(CT) do { if (mtt == 1) UOE_FOLD2(CT, 1); else if (mtt == 2) UOE_FOLD2(CT, 2); else if (mtt == 4) UOE_FOLD2(CT, 4); else UOE_FOLD2(CT, 8); } while (0)
            if (ct == 1) UOE_FOLD1(1);
            else if (mtt == 1) UOE_FOLD2(2, 1);
            else if (mtt == 2) UOE_FOLD2(2, 2);
            else UOE_FOLD2(2, 4);
#undef UOE_FOLD1
#undef UOE_FOLD2
#undef UOE_FOLD3
            if ((err = hipGetLastError()) != hipSuccess) return err;
            fold_ranges = fp.ranges;
        } else if (has_d) {
            const size_t shf = (((size_t)a.tc_d * a.m * 2 + 15) & ~(size_t)15) + (size_t)a.tc_d * a.n * sizeof(float) + 256 * 8 * sizeof(float);
            hipLaunchKernelGGL(route_fold_kernel, dim3(a.nchunks_d, a.b), dim3(256), shf, st, a);
            if ((err = hipGetLastError()) != hipSuccess) return err;
        }
    } else
    // one launch for both routers while x is small enough that the two do not simply queue up on HBM
    if (has_e && bf16 && data_mfma && (double)a.b * a.l * a.d * 2 <= 48e6) {
        const int n_data = a.nchunks_d * a.b;
        const dim3 grid(n_data + a.nchunks * groups_e);
        const size_t shd = data_mfma_lds(a.n, a.d, 4);
#define UOE_FUSED(RT, CT)                                                                                         \
    do {                                                                                                          \
        const size_t she = route_expert_mfma_lds<RT, CT>();                                                       \
        hipLaunchKernelGGL((route_expert_data_kernel<RT, CT>), grid, dim3(256), she > shd ? she : shd, st, a, n_data);   \
    } while (0)
        if (a.n <= 16) {
            if (rt == 4) UOE_FUSED(4, 1);
            else if (rt == 2) UOE_FUSED(2, 1);
            else UOE_FUSED(1, 1);
        } else {
            if (rt == 4) UOE_FUSED(4, 2);
            else if (rt == 2) UOE_FUSED(2, 2);
            else UOE_FUSED(1, 2);
        }
#undef UOE_FUSED
        if ((err = hipGetLastError()) != hipSuccess) return err;
    } else {
        if (has_e && bf16) {  // a.tc / a.nchunks follow route_expert_mfma_tokens_per_chunk
            const dim3 grid(a.nchunks, groups_e);
#define UOE_EXPERT(RT, CT) hipLaunchKernelGGL((route_expert_mfma_kernel<RT, CT>), grid, dim3(256), (route_expert_mfma_lds<RT, CT>()), st, a)
            if (a.n <= 16) {
                if (rt == 4) UOE_EXPERT(4, 1);
                else if (rt == 2) UOE_EXPERT(2, 1);
                else UOE_EXPERT(1, 1);
            } else {
                if (rt == 4) UOE_EXPERT(4, 2);
                else if (rt == 2) UOE_EXPERT(2, 2);
                else UOE_EXPERT(1, 2);
            }
#undef UOE_EXPERT
            if ((err = hipGetLastError()) != hipSuccess) return err;
        } else if (has_e) {
            if ((err = launch_partial_n<float>(a, true, false, st)) != hipSuccess) return err;
        }
        if (data_mfma) {
            const size_t sh = data_mfma_lds(a.n, a.d, 4);
            const dim3 grid(a.nchunks_d, a.b);
            if (a.n <= 16) hipLaunchKernelGGL((route_data_mfma_kernel<4, 1>), grid, dim3(256), sh, st, a);
            else hipLaunchKernelGGL((route_data_mfma_kernel<4, 2>), grid, dim3(256), sh, st, a);
            if ((err = hipGetLastError()) != hipSuccess) return err;
        } else if (has_d) {
            RouteArgs ad = a;  // the vector-ALU kernel takes its chunking from tc / nchunks
            ad.tc = a.tc_d;
            ad.nchunks = a.nchunks_d;
            err = bf16 ? launch_partial_n<bf16_t>(ad, false, true, st) : launch_partial_n<float>(ad, false, true, st);
            if (err != hipSuccess) return err;
        }
    }
    size_t sh = (size_t)a.m * (sizeof(float) + 1);
    const size_t stage_bytes = (size_t)a.n * a.m * sizeof(float);
    const bool staged = has_d && stage_bytes <= SELECT_STAGE_MAX;
    if (staged) sh = ((sh + 15) & ~(size_t)15) + stage_bytes;
    int fuse_reduce = staged && a.n * a.m <= SELECT_THREADS && (long)a.n * a.m * a.nchunks_d <= 16384;
    if (staged && fold_ranges > 0 && fold_ranges <= 16) fuse_reduce = 2;
    if (has_d && !fuse_reduce) {
        hipLaunchKernelGGL(route_reduce_kernel, dim3((a.n * a.m + 15) / 16, a.b), dim3(256), 0, st, a);
        err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    // rows other than 0 only produce patch lists and gates: skip them when neither is asked for
    const int rows = (a.patch_idx || a.patch_gate) ? a.n : 1;
    hipLaunchKernelGGL(route_select_kernel, dim3(rows, a.b), dim3(SELECT_THREADS), sh, st, a, (int)has_e,
                       (int)has_d, (int)staged, fuse_reduce);
    return hipGetLastError();
}

}  // namespace uoe

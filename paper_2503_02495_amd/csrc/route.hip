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

namespace uoe {

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
int route_data_tokens_per_chunk(int b, int l, int d, int n, bool bf16)
{
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
    const int n = a.n, d = a.d, l = a.l, m = a.m;
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

    // Fold with the chunk's rows of W_A: g[i][j] = sum_t t1[t][i] * W_A[t0 + t][j].  A thread owns
    // (token group tg, output group og): one expert i and VEC consecutive patches, for the tokens
    // tg, tg + TG, ...; the TG partial sums of an output are then added in group order.  (With few
    // outputs per sample, one thread per output would leave most of the workgroup idle behind a
    // serial walk over all the chunk's tokens.)
    const uint16_t *w_a = static_cast<const uint16_t *>(a.w_a);
    const int nm = n * m;
    float *gout = a.gpart + ((size_t)chunk * a.b + bb) * nm;
    const int vec = (m & 7) == 0 ? 8 : 1, mv = m / vec, og_n = n * mv;
    const int tg_n = og_n >= NTHREADS ? 1 : NTHREADS / og_n;
    float *part = t1s + TC * np;  // [tg_n][nm], at most NTHREADS * 8 floats
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
        if (fuse_reduce) {  // nm <= SELECT_THREADS: thread = (chunk group, value), groups summed in order
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

hipError_t launch_route(const RouteArgs &a, bool bf16, hipStream_t st)
{
    const bool has_e = a.w_e != nullptr, has_d = a.w_b != nullptr;
    hipError_t err = hipSuccess;
    const bool data_mfma = has_d && route_data_uses_mfma(a.b, a.l, a.d, a.n, bf16);
    const int rt = a.b > 32 ? 4 : (a.b > 16 ? 2 : 1);
    const int groups_e = (a.b + rt * 16 - 1) / (rt * 16);
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
    const bool fuse_reduce = staged && a.n * a.m <= SELECT_THREADS && (long)a.n * a.m * a.nchunks_d <= 16384;
    if (has_d && !fuse_reduce) {
        hipLaunchKernelGGL(route_reduce_kernel, dim3((a.n * a.m + 15) / 16, a.b), dim3(256), 0, st, a);
        err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    // rows other than 0 only produce patch lists and gates: skip them when neither is asked for
    const int rows = (a.patch_idx || a.patch_gate) ? a.n : 1;
    hipLaunchKernelGGL(route_select_kernel, dim3(rows, a.b), dim3(SELECT_THREADS), sh, st, a, (int)has_e,
                       (int)has_d, (int)staged, (int)fuse_reduce);
    return hipGetLastError();
}

}  // namespace uoe

// Routing of one block (Sec. III-B): expert-selection router (Eq. 21-22) and patch-wise
// data-selection router (Eq. 13, 14, 17).
//
// Three kernels:
//   route_partial : one pass over x.  A workgroup owns (chunk of tokens, sample); it streams the
//                   chunk of x once and, from the same registers, accumulates (a) the partial
//                   expert-router dot products against the matching chunk of W_E and (b) the
//                   per-token d->n map of the data router, which it then folds with the chunk's
//                   rows of W_A into a partial [n,m] logit tile.  HBM-bound: x and W_E are each
//                   read once (W_E chunks are shared by the b samples through L2).
//   route_reduce  : sums the per-chunk partials in fixed chunk order (deterministic).
//   route_select  : per sample: + noise, softmax over experts (Eq. 14 / 21), then top-c per
//                   expert and top-k per sample by rank counting: rank(j) = #{j' : g_j' > g_j or
//                   (g_j' == g_j and j' < j)}; keep rank < c.  The output slot of a kept index is
//                   the number of kept lower indices, so the list comes out ascending with no
//                   sort and ties go to the lower index by construction.
#include "common.h"

namespace uoe {

int route_tokens_per_chunk(int b, int l)
{
    // aim for >= ~1024 workgroups but keep a chunk within [16, 64] tokens
    long tc = ((long)b * l) / 1024;
    tc = (tc / 4) * 4;
    if (tc < 16) tc = 16;
    if (tc > 64) tc = 64;
    if (tc > l) tc = l;
    return (int)tc;
}

constexpr int ROUTE_THREADS = 256;
constexpr int ROUTE_WAVES = ROUTE_THREADS / 64;

template <typename T, int NMAX, bool HAS_E, bool HAS_D>
__global__ __launch_bounds__(ROUTE_THREADS) void route_partial_kernel(RouteArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int chunk = blockIdx.x, bb = blockIdx.y;
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

    const size_t ld = (size_t)l * d;
    for (int tl = wave; tl < tcur; tl += ROUTE_WAVES) {
        const int t = t0 + tl;
        const T *xr = x + ((size_t)bb * l + t) * d;
        float tacc[NMAX];
#pragma unroll
        for (int i = 0; i < NMAX; ++i) tacc[i] = 0.f;
        for (int e = lane * 8; e < d; e += 64 * 8) {
            float xv[8];
            load8(xr + e, xv);
#pragma unroll
            for (int i = 0; i < NMAX; ++i) {
                if (i < n) {
                    if (HAS_E) {
                        float wv[8];
                        load8(w_e + (size_t)i * ld + (size_t)t * d + e, wv);
#pragma unroll
                        for (int q = 0; q < 8; ++q) zacc[i] = fmaf(xv[q], wv[q], zacc[i]);
                    }
                    if (HAS_D) {
                        float wv[8];
                        load8(wb_t + i * d + e, wv);
#pragma unroll
                        for (int q = 0; q < 8; ++q) tacc[i] = fmaf(xv[q], wv[q], tacc[i]);
                    }
                }
            }
        }
        if (HAS_D) {
#pragma unroll
            for (int i = 0; i < NMAX; ++i) {
                if (i < n) {
                    const float s = wave_sum(tacc[i]);
                    if (lane == 0) t1s[tl * NMAX + i] = s;
                }
            }
        }
    }
    if (HAS_E) {
#pragma unroll
        for (int i = 0; i < NMAX; ++i) {
            if (i < n) {
                const float s = wave_sum(zacc[i]);
                if (lane == 0) zsh[wave * NMAX + i] = s;
            }
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

// sums partials over chunks in chunk order; one thread per reduced value
__global__ __launch_bounds__(256) void route_reduce_kernel(RouteArgs a, int has_e, int has_d)
{
    const long nz = has_e ? (long)a.b * a.n : 0;
    const long ng = has_d ? (long)a.b * a.n * a.m : 0;
    const long v = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (v < nz) {
        float s = 0.f;
        for (int ch = 0; ch < a.nchunks; ++ch) s += a.zpart[(size_t)ch * nz + v];
        a.zred[v] = s;
    } else if (v - nz < ng) {
        const long w = v - nz;
        float s = 0.f;
        for (int ch = 0; ch < a.nchunks; ++ch) s += a.gpart[(size_t)ch * ng + w];
        a.gred[w] = s;
    }
}

// One workgroup per sample.  LDS: gate tile [n*m] fp32 + kept flags [n*m] bytes.
__global__ __launch_bounds__(256) void route_select_kernel(RouteArgs a, int has_e, int has_d)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, bb = blockIdx.x;
    const int n = a.n, m = a.m, c = a.c, k = a.k, nm = n * m;
    float *g = reinterpret_cast<float *>(smem);
    unsigned char *kept = smem + (size_t)nm * sizeof(float);
    __shared__ float ge[32];
    __shared__ unsigned char ekept[32];

    // ---- data selection: Eq. 13 logits (+noise) -> Eq. 14 gate -> Eq. 17 top-c
    if (has_d) {
        for (int o = tid; o < nm; o += 256) {
            float v = a.gred[(size_t)bb * nm + o];
            if (a.noise_p) v += a.noise_p[(size_t)bb * nm + o];
            g[o] = v;
        }
        __syncthreads();
        for (int j = tid; j < m; j += 256) {  // softmax over the n experts of patch j
            float mx = -INFINITY;
            for (int i = 0; i < n; ++i) mx = fmaxf(mx, g[i * m + j]);
            float den = 0.f;
            for (int i = 0; i < n; ++i) den += expf(g[i * m + j] - mx);
            const float lden = logf(den);
            for (int i = 0; i < n; ++i) {
                const float sh = g[i * m + j] - mx;
                if (a.patch_gate) a.patch_gate[(size_t)bb * nm + i * m + j] = expf(sh) / den;
                // ranking key: the log of the gate.  Same order as the gate itself, but a gate too
                // small for fp32 keeps its rank instead of collapsing into a tie at zero.
                g[i * m + j] = sh - lden;
            }
        }
    } else {
        for (int o = tid; o < nm; o += 256) {
            g[o] = 0.0f;
            if (a.patch_gate) a.patch_gate[(size_t)bb * nm + o] = 1.0f;
        }
    }
    __syncthreads();
    for (int o = tid; o < nm; o += 256) {
        const int i = o / m, j = o - i * m;
        const float v = g[o];
        int rank = 0;
        for (int jj = 0; jj < m; ++jj) {
            const float w = g[i * m + jj];
            rank += (w > v || (w == v && jj < j)) ? 1 : 0;
        }
        kept[o] = rank < c;
    }
    __syncthreads();
    if (a.patch_idx) {
        for (int o = tid; o < nm; o += 256) {
            if (!kept[o]) continue;
            const int i = o / m, j = o - i * m;
            int pos = 0;
            for (int jj = 0; jj < j; ++jj) pos += kept[i * m + jj];
            a.patch_idx[((size_t)bb * n + i) * c + pos] = j;
        }
    }

    // ---- expert selection: Eq. 21 logits (+noise) -> softmax -> Eq. 22 top-k
    // The softmax is strictly increasing in the logit within a sample, so the k largest gates are
    // the k largest logits: rank on the logits, which cannot underflow.
    float z = 0.f;
    if (tid < n) {
        if (has_e) {
            z = a.zred[(size_t)bb * n + tid];
            if (a.noise_e) z += a.noise_e[(size_t)bb * n + tid];
        }
        ge[tid] = z;
    }
    __syncthreads();
    if (tid < n) {
        float gv = 1.0f;
        if (has_e) {
            float mx = -INFINITY;
            for (int i = 0; i < n; ++i) mx = fmaxf(mx, ge[i]);
            float den = 0.f;
            for (int i = 0; i < n; ++i) den += expf(ge[i] - mx);
            gv = expf(z - mx) / den;
        }
        if (a.expert_gate) a.expert_gate[(size_t)bb * n + tid] = gv;
        int rank = 0;
        for (int i = 0; i < n; ++i) rank += (ge[i] > z || (ge[i] == z && i < tid)) ? 1 : 0;
        ekept[tid] = rank < k;
    }
    __syncthreads();
    if (tid < n && ekept[tid] && a.expert_idx) {
        int pos = 0;
        for (int i = 0; i < tid; ++i) pos += ekept[i];
        a.expert_idx[(size_t)bb * k + pos] = tid;
    }
}

template <typename T, int NMAX>
static hipError_t launch_partial(const RouteArgs &a, bool has_e, bool has_d, hipStream_t st)
{
    dim3 grid(a.nchunks, a.b), block(ROUTE_THREADS);
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
    if (a.n <= 4) return launch_partial<T, 4>(a, has_e, has_d, st);
    if (a.n <= 8) return launch_partial<T, 8>(a, has_e, has_d, st);
    if (a.n <= 16) return launch_partial<T, 16>(a, has_e, has_d, st);
    return launch_partial<T, 32>(a, has_e, has_d, st);
}

hipError_t launch_route(const RouteArgs &a, bool bf16, hipStream_t st)
{
    const bool has_e = a.w_e != nullptr, has_d = a.w_b != nullptr;
    hipError_t err = hipSuccess;
    if (has_e || has_d) {
        err = bf16 ? launch_partial_n<bf16_t>(a, has_e, has_d, st) : launch_partial_n<float>(a, has_e, has_d, st);
        if (err != hipSuccess) return err;
        const long total = (has_e ? (long)a.b * a.n : 0) + (has_d ? (long)a.b * a.n * a.m : 0);
        hipLaunchKernelGGL(route_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, a,
                           (int)has_e, (int)has_d);
        err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    const size_t sh = (size_t)a.n * a.m * (sizeof(float) + 1);
    hipLaunchKernelGGL(route_select_kernel, dim3(a.b), dim3(256), sh, st, a, (int)has_e, (int)has_d);
    return hipGetLastError();
}

}  // namespace uoe

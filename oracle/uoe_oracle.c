/*
 * CPU fp64 oracle for the forward pass of one Union-of-Experts layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what
 * the layer computes, written from the paper (arXiv 2503.02495, Sec. III) in
 * the paper's order and notation.  It shares no code, header, table or helper
 * with the GPU library, and nothing in the product path may call it.
 *
 * Everything is `double`, row-major, with no intermediate rounding, no
 * blocking and no fusion: each function is the formula it cites, as loops.
 * The only liberty is `#pragma omp parallel for` over independent rows.
 *
 * Readings taken where the paper's text is silent or garbled (each also listed
 * in the design notes of the repository):
 *   - Eq. 13: FFN_B is a linear map d -> n applied per token, the result is
 *     transposed to [n, l], FFN_A is a linear map l -> m.  No bias, no
 *     activation (the only reading with g' in R^{n x m}).
 *   - Eq. 14: the softmax runs over the n experts for a fixed patch.
 *   - Eq. 17: top-c is taken on the gating VALUES of Eq. 14 (not the logits);
 *     ties go to the lower index; kept indices are then sorted ascending.
 *   - Eq. 21: one linear map R^{l*d} -> R^n on the flattened sample, g in
 *     R^{b x n}.
 *   - Eq. 22: kept expert indices are reported ascending.
 *   - Eq. 33: scores are Q K^T (row-vector convention), softmax along keys,
 *     scale 1/sqrt(d_h); attention runs jointly over the l_a = c*l_p selected
 *     tokens of one expert.
 *   - Eq. 39: the second MLP layer is linear (the activation sits only after
 *     the first layer), as the lossless split of Sec. III-A requires.
 *   - Eq. 20/26/36/40 add unweighted expert outputs; gate weighting is an
 *     option (flags below) and uses the softmax gate values un-renormalised.
 *   - Eq. 32 (Eq. 31 is a misprint of the perplexity formula): q' = [q^c, RoPE(q^r)],
 *     k' = [k^c, RoPE(k^r)]; the rotary part is the LAST rope_dim dims of a head, rotated in
 *     adjacent pairs (2i, 2i+1) by the angle p * 10000^(-2i/rope_dim), where p is the token's
 *     position in the COMPACTED sequence of its expert (0..l_a-1): Sec. III-B says selection keeps
 *     relative order while changing absolute position, and the shared mask of Fig. 4 treats the
 *     compacted sequence the same way.
 *   - Sec. III-C.3: the causal mask is the leading l_a x l_a lower-triangular block for every
 *     expert (key position <= query position in the compacted sequence); the padding mask is
 *     gathered with the same indices (Eq. 41) and removes padded KEYS from the softmax.  A query
 *     with no admissible key contributes nothing.
 *   - Both selections in one block (Sec. III-B, last paragraph): both routers
 *     read the block input; only patches selected by an ACTIVE expert are
 *     processed; the weight is the product of the two gates.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* contribution-weight / residual switches (values chosen by this file) */
#define ORACLE_RESIDUAL 1u     /* out = in + sum(...)   (Eq. 20/26); off: out = sum(...) */
#define ORACLE_GATE_EXPERT 2u  /* weight contributions by the Eq. 21 gate of the expert   */
#define ORACLE_GATE_PATCH 4u   /* weight contributions by the Eq. 14 gate of the patch    */
#define ORACLE_CAUSAL 8u       /* shared causal mask of Sec. III-C.3 (Fig. 4)             */

void uoe_oracle_set_threads(int t)
{
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

int uoe_oracle_get_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* C[M,N] = A[M,K] * B[K,N]; plain triple loop, rows independent. */
static void matmul(int M, int K, int N, const double *A, long lda, const double *B, long ldb,
                   double *C, long ldc)
{
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i) {
        double *Ci = C + (long)i * ldc;
        for (int j = 0; j < N; ++j) Ci[j] = 0.0;
        for (int kk = 0; kk < K; ++kk) {
            const double a = A[(long)i * lda + kk];
            const double *Bk = B + (long)kk * ldb;
            for (int j = 0; j < N; ++j) Ci[j] += a * Bk[j];
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Eq. 13: g'[b,i,j] = sum_t ( sum_e x[b,t,e] W_B[e,i] ) W_A[t,j]  (+ noise)  */
/* x [b,l,d]; W_B [d,n]; W_A [l,m]; noise [b,n,m] or NULL; gprime [b,n,m].    */
void uoe_oracle_data_router_logits(int b, int l, int d, int n, int m, const double *x,
                                   const double *W_B, const double *W_A, const double *noise,
                                   double *gprime)
{
    double *t1 = (double *)malloc(sizeof(double) * (size_t)l * n); /* FFN_B(x): [l,n] */
    for (int bb = 0; bb < b; ++bb) {
        matmul(l, d, n, x + (long)bb * l * d, d, W_B, n, t1, n);
        /* FFN_A applied to the transpose: g'[i,j] = sum_t t1[t,i] W_A[t,j] */
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < m; ++j) {
                double s = 0.0;
                for (int t = 0; t < l; ++t) s += t1[(long)t * n + i] * W_A[(long)t * m + j];
                if (noise) s += noise[((long)bb * n + i) * m + j];
                gprime[((long)bb * n + i) * m + j] = s;
            }
    }
    free(t1);
}

/* Eq. 14: g[b,i,j] = exp(g'[b,i,j]) / sum_t exp(g'[b,t,j]), t over the n experts. */
void uoe_oracle_patch_gate(int b, int n, int m, const double *gprime, double *g)
{
    for (int bb = 0; bb < b; ++bb)
        for (int j = 0; j < m; ++j) {
            double mx = -INFINITY, den = 0.0;
            for (int i = 0; i < n; ++i) {
                double v = gprime[((long)bb * n + i) * m + j];
                if (v > mx) mx = v;
            }
            for (int i = 0; i < n; ++i) den += exp(gprime[((long)bb * n + i) * m + j] - mx);
            for (int i = 0; i < n; ++i)
                g[((long)bb * n + i) * m + j] = exp(gprime[((long)bb * n + i) * m + j] - mx) / den;
        }
}

/* Topk of Eq. 17 / Eq. 22 on one row of `count` values: order indices by
 * (value descending, index ascending), keep the first `keep`, report them in
 * ascending index order.  margin = |a-b| / max(|a|,|b|) between the last kept
 * and the first dropped value (the near-tie measure), or -1 when nothing is
 * dropped. */
static void top_select(const double *v, int count, int keep, int32_t *out, double *margin)
{
    int *ord = (int *)malloc(sizeof(int) * (size_t)count);
    for (int j = 0; j < count; ++j) { /* insertion sort by (-v, j) */
        int p = j;
        while (p > 0 && v[ord[p - 1]] < v[j]) { /* strict: equal values keep index order */
            ord[p] = ord[p - 1];
            --p;
        }
        ord[p] = j;
    }
    if (margin) {
        if (keep < count) {
            double a = v[ord[keep - 1]], bb = v[ord[keep]];
            double den = fmax(fabs(a), fabs(bb));
            *margin = den > 0.0 ? fabs(a - bb) / den : 0.0;
        } else
            *margin = -1.0;
    }
    /* the kept indices are reported in ascending order (Sec. III-B, the text after Eq. 17) */
    for (int a = 0; a < keep; ++a) {
        int p = a;
        int val = ord[a];
        while (p > 0 && out[p - 1] > val) {
            out[p] = out[p - 1];
            --p;
        }
        out[p] = val;
    }
    free(ord);
}

/* Eq. 17 for every (sample, expert): id[b,i,0..c) ascending; margin[b,i]. */
void uoe_oracle_top_c(int b, int n, int m, int c, const double *g, int32_t *id, double *margin)
{
    for (long r = 0; r < (long)b * n; ++r)
        top_select(g + r * m, m, c, id + r * c, margin ? margin + r : NULL);
}

/* Eq. 21: z[b,i] = sum_{t,e} x[b,t,e] W_E[i, t*d+e] (+ noise); g = softmax_i z. */
/* x [b, l*d]; W_E [n, l*d]; noise [b,n] or NULL; z, g [b,n].                    */
void uoe_oracle_expert_router(int b, long ld, int n, const double *x, const double *W_E,
                              const double *noise, double *z, double *g)
{
    for (int bb = 0; bb < b; ++bb) {
#pragma omp parallel for schedule(static)
        for (int i = 0; i < n; ++i) {
            double s = 0.0;
            for (long q = 0; q < ld; ++q) s += x[(long)bb * ld + q] * W_E[(long)i * ld + q];
            if (noise) s += noise[(long)bb * n + i];
            z[(long)bb * n + i] = s;
        }
        double mx = -INFINITY, den = 0.0;
        for (int i = 0; i < n; ++i)
            if (z[(long)bb * n + i] > mx) mx = z[(long)bb * n + i];
        for (int i = 0; i < n; ++i) den += exp(z[(long)bb * n + i] - mx);
        for (int i = 0; i < n; ++i) g[(long)bb * n + i] = exp(z[(long)bb * n + i] - mx) / den;
    }
}

/* Eq. 22 for every sample: id[b,0..k) ascending; margin[b]. */
void uoe_oracle_top_k(int b, int n, int k, const double *g, int32_t *id, double *margin)
{
    for (long r = 0; r < b; ++r) top_select(g + r * n, n, k, id + r * k, margin ? margin + r : NULL);
}

/* Eq. 23: id^(i) = { j in [0,b) : i in id'_j }, ascending.  counts[n], lists[n*b]
 * (row i holds counts[i] valid entries). */
void uoe_oracle_expert_lists(int b, int n, int k, const int32_t *id, int32_t *counts, int32_t *lists)
{
    for (int i = 0; i < n; ++i) {
        counts[i] = 0;
        for (int j = 0; j < b; ++j)
            for (int s = 0; s < k; ++s)
                if (id[(long)j * k + s] == i) lists[(long)i * b + counts[i]++] = j;
    }
}

/* ------------------------------------------------------------------------- */
/* Eq. 32: rotate the last rope_dim dims of every row of X [rows, d_h]; row r is at position r. */
static void rope_rows(double *X, int rows, int d_h, int rope_dim)
{
    const int first = d_h - rope_dim;
    for (int r = 0; r < rows; ++r)
        for (int i = 0; i < rope_dim / 2; ++i) {
            const double theta = pow(10000.0, -2.0 * i / rope_dim);
            const double cs = cos(r * theta), sn = sin(r * theta);
            double *p = X + (long)r * d_h + first + 2 * i;
            const double a = p[0], b = p[1];
            p[0] = a * cs - b * sn;
            p[1] = a * sn + b * cs;
        }
}

/* Selective Multi-Head Attention, Eq. 27-36, with the optional partial RoPE of Eq. 32 and the
 * masks of Sec. III-C.3.
 * x [b,l,d]; Wq,Wk,Wv [n,d,d_h]; Wo [n,d_h,d]; expert_id [b,k] (Eq. 22);
 * gE [b,n] (Eq. 21); patch_id [b,n,c] (Eq. 17); gD [b,n,m] (Eq. 14); u [b,l,d];
 * rope_dim even, 0 = none; pad_mask [b,l] bytes (1 = token, 0 = padding) or NULL. */
void uoe_oracle_smha(int b, int l, int d, int n, int k, int m, int c, int d_h, unsigned flags,
                     const double *x, const double *Wq, const double *Wk, const double *Wv,
                     const double *Wo, const int32_t *expert_id, const double *gE,
                     const int32_t *patch_id, const double *gD, int rope_dim,
                     const unsigned char *pad_mask, double *u)
{
    const int l_p = l / m, l_a = c * l_p;
    double *H = (double *)malloc(sizeof(double) * (size_t)l_a * d);
    double *Q = (double *)malloc(sizeof(double) * (size_t)l_a * d_h);
    double *K = (double *)malloc(sizeof(double) * (size_t)l_a * d_h);
    double *V = (double *)malloc(sizeof(double) * (size_t)l_a * d_h);
    double *S = (double *)malloc(sizeof(double) * (size_t)l_a * l_a);
    double *O = (double *)malloc(sizeof(double) * (size_t)l_a * d_h);
    double *U = (double *)malloc(sizeof(double) * (size_t)l_a * d);
    int *T = (int *)malloc(sizeof(int) * (size_t)l_a);
    const double scale = 1.0 / sqrt((double)d_h);

    for (int bb = 0; bb < b; ++bb) {
        const double *xb = x + (long)bb * l * d;
        double *ub = u + (long)bb * l * d;
        /* selective residual: u starts as h (or as zero when the residual is off) */
        for (long q = 0; q < (long)l * d; ++q) ub[q] = (flags & ORACLE_RESIDUAL) ? xb[q] : 0.0;

        for (int s = 0; s < k; ++s) {
            const int i = expert_id[(long)bb * k + s]; /* an active expert of this sample */
            const int32_t *idi = patch_id + ((long)bb * n + i) * c;
            /* Eq. 12 + 18: token positions of the selected patches, in order */
            for (int t = 0; t < c; ++t)
                for (int r = 0; r < l_p; ++r) T[t * l_p + r] = idi[t] * l_p + r;
            for (int r = 0; r < l_a; ++r) memcpy(H + (long)r * d, xb + (long)T[r] * d, sizeof(double) * d);
            /* Eq. 28-30 */
            matmul(l_a, d, d_h, H, d, Wq + (long)i * d * d_h, d_h, Q, d_h);
            matmul(l_a, d, d_h, H, d, Wk + (long)i * d * d_h, d_h, K, d_h);
            matmul(l_a, d, d_h, H, d, Wv + (long)i * d * d_h, d_h, V, d_h);
            /* Eq. 32 */
            if (rope_dim > 0) {
                rope_rows(Q, l_a, d_h, rope_dim);
                rope_rows(K, l_a, d_h, rope_dim);
            }
            /* Eq. 33: s = softmax(q k^T / sqrt(d_h)) along the admissible keys */
#pragma omp parallel for schedule(static)
            for (int r = 0; r < l_a; ++r) {
                double *Sr = S + (long)r * l_a;
                double mx = -INFINITY, den = 0.0;
                for (int j = 0; j < l_a; ++j) {
                    int ok = 1;
                    if ((flags & ORACLE_CAUSAL) && j > r) ok = 0;                    /* Fig. 4 */
                    if (pad_mask && !pad_mask[(long)bb * l + T[j]]) ok = 0;          /* Eq. 41 */
                    if (!ok) {
                        Sr[j] = -INFINITY;
                        continue;
                    }
                    double a = 0.0;
                    for (int e = 0; e < d_h; ++e) a += Q[(long)r * d_h + e] * K[(long)j * d_h + e];
                    Sr[j] = a * scale;
                    if (Sr[j] > mx) mx = Sr[j];
                }
                for (int j = 0; j < l_a; ++j) {
                    Sr[j] = (Sr[j] == -INFINITY) ? 0.0 : exp(Sr[j] - mx);
                    den += Sr[j];
                }
                for (int j = 0; j < l_a; ++j) Sr[j] = den > 0.0 ? Sr[j] / den : 0.0;
            }
            /* Eq. 34, Eq. 35 */
            matmul(l_a, l_a, d_h, S, l_a, V, d_h, O, d_h);
            matmul(l_a, d_h, d, O, d_h, Wo + (long)i * d_h * d, d, U, d);
            /* Eq. 36: index add at the positions the rows came from */
            for (int r = 0; r < l_a; ++r) {
                double w = 1.0;
                if (flags & ORACLE_GATE_EXPERT) w *= gE[(long)bb * n + i];
                if (flags & ORACLE_GATE_PATCH) w *= gD[((long)bb * n + i) * m + idi[r / l_p]];
                for (int e = 0; e < d; ++e) ub[(long)T[r] * d + e] += w * U[(long)r * d + e];
            }
        }
    }
    free(H); free(Q); free(K); free(V); free(S); free(O); free(U); free(T);
}

/* ------------------------------------------------------------------------- */
/* Union-of-MLP-Experts in expert-selection mode, Eq. 38-40 with Eq. 24-26.
 * u [b,l,d]; A_I [n,d,d_e]; A_O [n,d_e,d]; expert_id [b,k]; gE [b,n]; h [b,l,d]. */
void uoe_oracle_uome(int b, int l, int d, int n, int k, int d_e, unsigned flags, const double *u,
                     const double *A_I, const double *A_O, const int32_t *expert_id,
                     const double *gE, double *h)
{
    double *Vh = (double *)malloc(sizeof(double) * (size_t)l * d_e);
    double *Hp = (double *)malloc(sizeof(double) * (size_t)l * d);
    for (int bb = 0; bb < b; ++bb) {
        const double *ub = u + (long)bb * l * d;
        double *hb = h + (long)bb * l * d;
        for (long q = 0; q < (long)l * d; ++q) hb[q] = (flags & ORACLE_RESIDUAL) ? ub[q] : 0.0;
        for (int s = 0; s < k; ++s) {
            const int i = expert_id[(long)bb * k + s];
            /* Eq. 38: v_i = SiLU(u A^I_i) */
            matmul(l, d, d_e, ub, d, A_I + (long)i * d * d_e, d_e, Vh, d_e);
            for (long q = 0; q < (long)l * d_e; ++q) Vh[q] = Vh[q] / (1.0 + exp(-Vh[q]));
            /* Eq. 39 (linear second layer): h'_i = v_i A^O_i */
            matmul(l, d_e, d, Vh, d_e, A_O + (long)i * d_e * d, d, Hp, d);
            /* Eq. 40 / 26: index add of the expert's output onto its sample */
            const double w = (flags & ORACLE_GATE_EXPERT) ? gE[(long)bb * n + i] : 1.0;
            for (long q = 0; q < (long)l * d; ++q) hb[q] += w * Hp[q];
        }
    }
    free(Vh); free(Hp);
}

/* ------------------------------------------------------------------------- */
/* Union-of-MLP-Experts with patch-wise data selection (Eq. 37-40 in full: u' = f_DS(u) per expert).
 * Expert i of an active slot sees only its c selected patches (ascending, as routing returns
 * them): u'_i [l_a,d] gathered (Eq. 18), v_i = SiLU(u'_i A^I_i) (Eq. 38), h'_i = v_i A^O_i
 * (Eq. 39, linear second layer), and the rows of h'_i are index-added onto the tokens they were
 * gathered from (Eq. 40), weighted by the expert gate and/or the patch gate as the flags say.
 * u [b,l,d]; A_I [n,d,d_e]; A_O [n,d_e,d]; expert_id [b,k]; gE [b,n]; patch_id [b,n,c];
 * gD [b,n,m]; h [b,l,d]. */
void uoe_oracle_uome_ds(int b, int l, int d, int n, int k, int m, int c, int d_e, unsigned flags,
                        const double *u, const double *A_I, const double *A_O,
                        const int32_t *expert_id, const double *gE, const int32_t *patch_id,
                        const double *gD, double *h)
{
    const int l_p = l / m, l_a = c * l_p;
    double *Up = (double *)malloc(sizeof(double) * (size_t)l_a * d);
    double *Vh = (double *)malloc(sizeof(double) * (size_t)l_a * d_e);
    double *Hp = (double *)malloc(sizeof(double) * (size_t)l_a * d);
    for (int bb = 0; bb < b; ++bb) {
        const double *ub = u + (long)bb * l * d;
        double *hb = h + (long)bb * l * d;
        for (long q = 0; q < (long)l * d; ++q) hb[q] = (flags & ORACLE_RESIDUAL) ? ub[q] : 0.0;
        for (int s = 0; s < k; ++s) {
            const int i = expert_id[(long)bb * k + s];
            const int32_t *pid = patch_id + ((long)bb * n + i) * c;
            /* Eq. 18: the expert's patches, in the order routing returned them */
            for (int t = 0; t < c; ++t)
                for (int r = 0; r < l_p; ++r)
                    for (int e = 0; e < d; ++e)
                        Up[((long)t * l_p + r) * d + e] = ub[((long)pid[t] * l_p + r) * d + e];
            matmul(l_a, d, d_e, Up, d, A_I + (long)i * d * d_e, d_e, Vh, d_e);
            for (long q = 0; q < (long)l_a * d_e; ++q) Vh[q] = Vh[q] / (1.0 + exp(-Vh[q]));
            matmul(l_a, d_e, d, Vh, d_e, A_O + (long)i * d_e * d, d, Hp, d);
            for (int t = 0; t < c; ++t) {
                double w = 1.0;
                if (flags & ORACLE_GATE_EXPERT) w *= gE[(long)bb * n + i];
                if (flags & ORACLE_GATE_PATCH) w *= gD[((long)bb * n + i) * m + pid[t]];
                for (int r = 0; r < l_p; ++r)
                    for (int e = 0; e < d; ++e)
                        hb[((long)pid[t] * l_p + r) * d + e] += w * Hp[((long)t * l_p + r) * d + e];
            }
        }
    }
    free(Up); free(Vh); free(Hp);
}

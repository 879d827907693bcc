/*
 * uoe.h -- C ABI of the MI355X (gfx950) forward pass of one Union-of-Experts layer
 * (arXiv 2503.02495, Sec. III), and of its backward pass.
 *
 * Notation is the paper's: b batch, l sequence length, d model dim, n experts,
 * k experts kept per sample, m patches per sample, l_p = l/m tokens per patch,
 * c patches kept per expert, l_a = c*l_p tokens one attention expert sees,
 * `width` = d_h (SMHA head-expert dim) or d_e (UoME expert hidden dim).
 *
 * Conventions for every call
 *   - All tensor pointers are DEVICE pointers owned by the caller, row-major,
 *     contiguous, 16-byte aligned.  The library allocates no device memory,
 *     keeps no state between calls and never retains a pointer.  Scratch space
 *     is the caller's `ws` buffer of at least uoe_workspace_bytes() bytes (the
 *     backward calls have sizing functions of their own).
 *   - Calls only enqueue work on `hip_stream` (a hipStream_t passed as void*;
 *     NULL = the default stream) and return without waiting.  Calls on distinct
 *     streams with distinct workspaces may run concurrently.
 *   - Return value: a uoe_status.  Argument validation happens first, on the
 *     host, and touches no device state; a rejected call has launched nothing.
 *     No exceptions, no abort, nothing printed.
 *   - Storage dtype (x, weights, outputs) is fp32 or bf16; all accumulation is
 *     fp32; gates are fp32; indices are int32.
 *   - Inputs must be finite; behaviour on NaN/Inf is unspecified.
 *   - Environment: UOE_ROUTE_STREAM_MIN_BYTES (read at every routing call) moves the input size, in
 *     bytes of x plus the expert router's weights, from which the routers run as one streaming
 *     pass over x (default 100e6; 0 = whenever that kernel applies).  Results do not depend on it
 *     beyond the summation order of the router logits.  UOE_STREAM_ONCE_MIN_BYTES (read at every call)
 *     moves the tensor size, in bytes, from which outputs that a call writes once and residuals at
 *     their last use are accessed with the non-temporal hint (default 48 MiB; 0 = always).  Results
 *     do not depend on it at all.
 *   - Shape limits, all checked on the host before anything is launched (a valid request outside
 *     them returns UOE_ERR_UNSUPPORTED): d % 8 == 0, width % 8 == 0, l % m == 0, 1 <= n <= 32,
 *     1 <= k <= n, 1 <= c <= m, m <= 1024, n*m <= 8192, width <= 128 for SMHA, b*m <= 65535 and
 *     b*k <= 65535 (grid dimensions), b*l*max(d, k*width) <= 1e12 (index arithmetic), and with a
 *     data router n*d*sizeof(element) <= 48 KiB (W_B is staged in LDS).  Also UNSUPPORTED:
 *     UOE_FLAG_CAUSAL or rope_dim on a UoME call (uoe_route and uoe_gather ignore them).
 *   - Routing indices (expert_idx, patch_idx) handed to a compute call are caller data: an index
 *     outside [0, n) or [0, m) is clamped into range (the call then works on the wrong row, but never
 *     outside a tensor); it is not reported.
 */
#ifndef UOE_H
#define UOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    UOE_OK = 0,
    UOE_ERR_INVALID_ARG = 1, /* NULL where not allowed, bad sizes, misaligned pointer, aliasing   */
    UOE_ERR_UNSUPPORTED = 2, /* a valid request outside this build (see shape limits, flags)      */
    UOE_ERR_WORKSPACE = 3,   /* ws is NULL or ws_bytes is below uoe_workspace_bytes()             */
    UOE_ERR_DEVICE = 4,      /* a kernel launch was refused by the runtime                        */
    UOE_ERR_SCRATCH_LIMIT = 5 /* uoe_route_static: the request needs more than its fixed scratch  */
} uoe_status;

enum { UOE_F32 = 0, UOE_BF16 = 1 }; /* storage dtype of activations, weights and outputs */

enum {
    UOE_FLAG_RESIDUAL = 1u << 0,    /* out = in + sum(...)  (Eq. 20/26/36/40); off: out = sum(...)  */
    UOE_FLAG_GATE_EXPERT = 1u << 1, /* weight an expert's contribution by its Eq. 21 gate g[b,i]    */
    UOE_FLAG_GATE_PATCH = 1u << 2,  /* weight a patch's contribution by its Eq. 14 gate g[b,i,j]    */
    UOE_FLAG_CAUSAL = 1u << 3       /* SMHA only: shared causal mask of Sec. III-C.3 / Fig. 4       */
};

/* One block (SMHA or UoME) of the layer. */
typedef struct {
    int32_t b, l, d;     /* batch, sequence length, model dim                                        */
    int32_t n, k;        /* experts; experts kept per sample (k == n: expert selection off)          */
    int32_t m, c;        /* patches per sample; patches kept per expert (c == m: data selection off) */
    int32_t width;       /* d_h (SMHA) or d_e (UoME)                                                  */
    int32_t dtype;       /* UOE_F32 | UOE_BF16                                                        */
    uint32_t flags;      /* UOE_FLAG_*                                                                */
    int32_t rope_dim;    /* SMHA only: rotary dims at the end of each head (Eq. 32); even, 0 = none   */
    int32_t reserved[5]; /* must be 0                                                                 */
} uoe_block_desc;

/* Bytes of workspace that any call on these blocks needs (either may be NULL).
 * Returns 0 if a given descriptor is invalid. */
size_t uoe_workspace_bytes(const uoe_block_desc *smha, const uoe_block_desc *uome);

/* Static text for a uoe_status value. */
const char *uoe_status_string(int status);

/*
 * Routing of one block (Sec. III-B): expert selection, Eq. 21-22, and
 * patch-wise data selection, Eq. 13, 14 and 17, both reading the block input x.
 *
 *   x            [b,l,d]   block input (device, dtype)
 *   w_expert     [n, l*d]  expert router weights; NULL iff k == n and the gate is to be 1
 *   w_b, w_a     [d,n], [l,m]  data router: per-token map d->n, then map l->m over the
 *                          transposed result (Eq. 13); both NULL iff c == m and gate 1
 *   noise_expert [b,n] fp32, noise_patch [b,n,m] fp32: optional additive logit noise, or NULL
 * Outputs (device, caller-owned; each may be NULL, and what it would hold is then not written: a
 * call with every output NULL computes nothing useful but is valid):
 *   expert_idx   [b,k] int32   the k experts with the largest gate, ascending index;
 *                              ties go to the lower index
 *   expert_gate  [b,n] fp32    softmax over experts of the Eq. 21 logits
 *   patch_idx    [b,n,c] int32 for EVERY expert the c patches with the largest Eq. 14 gate
 *                              (ranked on the gate value, not the logit), ascending index
 *   patch_gate   [b,n,m] fp32  Eq. 14: softmax over the n experts for each patch
 * For a UoME block in expert-selection mode pass m = c = 1 and w_b = w_a = NULL.
 */
int uoe_route(const uoe_block_desc *blk, const void *x, const void *w_expert, const void *w_b,
              const void *w_a, const float *noise_expert, const float *noise_patch,
              int32_t *expert_idx, float *expert_gate, int32_t *patch_idx, float *patch_gate,
              void *ws, size_t ws_bytes, void *hip_stream);

/*
 * uoe_route for callers that cannot allocate or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  Same arguments, outputs, kernels
 * and results as uoe_route, without ws / ws_bytes: the per-chunk partial sums of the routers live
 * in a fixed array of UOE_ROUTE_STATIC_SCRATCH_BYTES in device memory that is part of the library
 * image (one copy per GPU, held until the process ends; its address is looked up on the first
 * call on each device).  The call allocates nothing, on the host or on the device.
 *   - A descriptor whose partial sums need more than that (what uoe_workspace_bytes counts for
 *     routing: about 4*(chunks*b*n*(m+1) + b*n*m) bytes with up to 512 chunks) is rejected with
 *     UOE_ERR_SCRATCH_LIMIT and nothing is launched.  The five workload shapes need at most 6.3 MiB
 *     (the largest one, whose routers run as one streaming pass, keeps a [b,l,n] fp32 array there).
 *   - The device of hip_stream must be the current device.
 *   - All calls on one GPU share the array: calls that overlap in time on one GPU (different
 *     streams or threads) race and give wrong results; calls on one stream are safe back to back.
 *     Every value the kernels read from the array was written earlier by the same call, so nothing
 *     needs to be cleared between calls.
 */
enum { UOE_ROUTE_STATIC_SCRATCH_BYTES = 8 * 1024 * 1024 };
int uoe_route_static(const uoe_block_desc *blk, const void *x, const void *w_expert, const void *w_b,
                     const void *w_a, const float *noise_expert, const float *noise_patch,
                     int32_t *expert_idx, float *expert_gate, int32_t *patch_idx, float *patch_gate,
                     void *hip_stream);

/*
 * Dynamic capacity of the two-stage routing (Eq. 15-16) and the statistics of the balance loss
 * (Eq. 43-44), from the block's data router alone.  Stage 1: every patch names its patch_k experts
 * with the highest Eq. 14 gate (ties to the lower expert index); count[b,i] = number of patches
 * that named expert i; capacity[b] = max_i count[b,i] (Eq. 16, per sample);
 * load_f[b,i] = n * count[b,i] / (patch_k * m) (Eq. 43 with the patch as the routed unit);
 * load_p[b,i] = mean over patches of the gate (Eq. 44).
 * A caller that wants the paper's dynamic allocation reads capacity back, takes c = the largest
 * value over the batch (one c per call: the selected sequences of a batch share their length) and
 * calls uoe_route / uoe_smha_forward with that c in the descriptor: c is a run-time value there.
 *   x, w_b, w_a, noise_patch as for uoe_route (blk->k and blk->c are not used); 1 <= patch_k <= n
 *   capacity [b] int32 (device); load_f, load_p [b,n] fp32 (device) or NULL
 *   n*m <= 8192 (the logits of a sample are held in LDS), else UOE_ERR_UNSUPPORTED
 */
int uoe_route_capacity(const uoe_block_desc *blk, const void *x, const void *w_b, const void *w_a,
                       const float *noise_patch, int32_t patch_k, int32_t *capacity, float *load_f,
                       float *load_p, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * The auxiliary load-balancing loss (Eq. 42) from the statistics uoe_route_capacity returns, and
 * its gradient with respect to the patch gates:
 *   loss[b] = alpha * sum_i load_f[b,i] * load_p[b,i]                       (one value per sequence)
 *   d_patch_gate[b,i,j] += alpha * load_f[b,i] / m                          (every patch j)
 * load_f counts selections and is piecewise constant, so only load_p = mean_j gate[b,i,j] (Eq. 44)
 * passes a gradient.  d_patch_gate [b,n,m] fp32 is UPDATED in place (it holds the block's own gate
 * gradient, as uoe_smha_backward returns it, and goes on to uoe_route_backward); NULL = loss only.
 * loss [b] fp32 may be NULL when only the gradient is wanted.  fp32 arithmetic; blk gives b, n, m.
 */
int uoe_balance_loss(const uoe_block_desc *blk, const float *load_f, const float *load_p,
                     float alpha, float *loss, float *d_patch_gate, void *hip_stream);

/*
 * Index selection of Eq. 18 / 24 as a standalone copy: for every active unit
 * (sample b, slot s < k, expert i = expert_idx[b,s]) the l_a selected token rows
 * of x, in ascending position, into h[b,s,:,:].
 *   h   [b,k,l_a,d]  (device, dtype).  Needs no workspace.
 * (The SMHA call below does this selection inside its projection kernel; this
 * entry point exists for callers that want the compacted buffer itself.)
 */
int uoe_gather(const uoe_block_desc *blk, const void *x, const int32_t *expert_idx,
               const int32_t *patch_idx, void *h, void *hip_stream);

/*
 * Selective Multi-Head Attention on given routing results (Eq. 27-36):
 * for every active unit gather its l_a tokens, project with W^q_i, W^k_i, W^v_i
 * (Eq. 28-30), softmax(q k^T / sqrt(d_h)) v jointly over the l_a tokens
 * (Eq. 33-34), project with W^o_i (Eq. 35), and add the rows back at the
 * positions they came from (Eq. 36), weighted per the gate flags.
 *   wq, wk, wv [n,d,d_h]; wo [n,d_h,d]; routing tensors as written by uoe_route
 *   (expert_gate / patch_gate may be NULL when the matching gate flag is off)
 *   out [b,l,d] must not alias x.  Rows of patches no active expert selected are
 *   x (or 0 without UOE_FLAG_RESIDUAL) exactly.  Deterministic: no atomics.
 * Optional (Sec. III-C.1/3):
 *   blk->rope_dim > 0   partial RoPE (Eq. 32): the last rope_dim dims of each head of q and k are
 *                       rotated in adjacent pairs (2i, 2i+1) by position * 10000^(-2i/rope_dim); the
 *                       position of a token is its index in its expert's compacted sequence
 *   UOE_FLAG_CAUSAL     every expert uses the leading l_a x l_a lower-triangular mask: key
 *                       position <= query position in the compacted sequence (Fig. 4)
 * A query row with no admissible key contributes nothing.
 */
int uoe_smha_forward(const uoe_block_desc *blk, const void *x, const void *wq, const void *wk,
                     const void *wv, const void *wo, const int32_t *expert_idx,
                     const float *expert_gate, const int32_t *patch_idx, const float *patch_gate,
                     void *out, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * uoe_smha_forward with a padding mask (Eq. 41): pad_mask [b,l] bytes on the device, 1 = token,
 * 0 = padding, gathered with each expert's indices; padded KEYS are removed from the softmax
 * (rows of padded queries are still computed).  pad_mask == NULL is uoe_smha_forward.
 */
int uoe_smha_forward_masked(const uoe_block_desc *blk, const void *x, const void *wq, const void *wk,
                            const void *wv, const void *wo, const int32_t *expert_idx,
                            const float *expert_gate, const int32_t *patch_idx, const float *patch_gate,
                            const uint8_t *pad_mask, void *out, void *ws, size_t ws_bytes,
                            void *hip_stream);

/*
 * The steps of uoe_smha_forward_masked one at a time, for callers that time or inspect them
 * (Eq. 28-30 + Eq. 32; Eq. 33-34; Eq. 35-36).  `steps` is a non-empty set of UOE_SMHA_STEP_* bits;
 * the selected steps run in their natural order on the same workspace, and a step reads what the
 * steps before it left there (q, k, v; the attention output), by this call or by an earlier one
 * with the same descriptor, routing and ws.  `out` is only written by UOE_SMHA_STEP_OUT.  All bits
 * set is uoe_smha_forward_masked.  Same arguments, limits and errors otherwise.
 */
enum { UOE_SMHA_STEP_QKV = 1u, UOE_SMHA_STEP_ATTENTION = 2u, UOE_SMHA_STEP_OUT = 4u };
int uoe_smha_forward_steps(const uoe_block_desc *blk, const void *x, const void *wq, const void *wk,
                           const void *wv, const void *wo, const int32_t *expert_idx,
                           const float *expert_gate, const int32_t *patch_idx, const float *patch_gate,
                           const uint8_t *pad_mask, void *out, void *ws, size_t ws_bytes, uint32_t steps,
                           void *hip_stream);

/*
 * Union-of-MLP-Experts on given routing results (Eq. 37-40).  The second layer is linear.
 *   a_in [n,d,d_e]; a_out [n,d_e,d]; expert_idx [b,k]; expert_gate [b,n] or NULL
 * Expert-selection mode (patch_idx NULL; needs blk->c == blk->m and no UOE_FLAG_GATE_PATCH, with
 * Eq. 24-26): out[b] = u[b] + sum over the sample's k experts of gate * SiLU(u[b] A^I_i) A^O_i.
 * Data-selection mode (patch_idx [b,n,c] given, ascending per (b,i); Eq. 37 with Eq. 12-18):
 * active expert i processes only the tokens of its c selected patches, and its rows are added
 * back onto those tokens, weighted by expert_gate[b,i] and/or patch_gate[b,i,patch] as the flags
 * say (patch_gate [b,n,m], required with UOE_FLAG_GATE_PATCH).  Tokens nobody selected keep the
 * residual only.  Wrong pointer combinations: UOE_ERR_INVALID_ARG.
 *   out [b,l,d] must not alias u.  Deterministic: no atomics.
 */
int uoe_uome_forward(const uoe_block_desc *blk, const void *u, const void *a_in, const void *a_out,
                     const int32_t *expert_idx, const float *expert_gate, const int32_t *patch_idx,
                     const float *patch_gate, void *out, void *ws, size_t ws_bytes,
                     void *hip_stream);

/*
 * The two contractions of uoe_uome_forward as separate calls (same kernels), for callers that
 * keep the hidden activations or time the steps one by one.
 *   uoe_uome_up   (Eq. 38): hidden[b,l,s*d_e + j] = gate * SiLU(u[b] A^I_i)[.,j] for the sample's
 *                 s-th active expert i = expert_idx[b,s]; hidden is [b,l,k*d_e] in the storage
 *                 dtype, written in full.  expert_gate may be NULL without UOE_FLAG_GATE_EXPERT.
 *   uoe_uome_down (Eq. 39-40): out[b] = (u[b] +) hidden[b] * [A^O_i rows of the active experts,
 *                 stacked]; out must not alias u or hidden.
 * Neither needs a workspace.
 */
int uoe_uome_up(const uoe_block_desc *blk, const void *u, const void *a_in, const int32_t *expert_idx,
                const float *expert_gate, void *hidden, void *hip_stream);
int uoe_uome_down(const uoe_block_desc *blk, const void *hidden, const void *a_out, const void *u,
                  const int32_t *expert_idx, void *out, void *hip_stream);

/*
 * Backward pass of uoe_uome_forward (the derivatives of Eq. 37-40; the selections of Eq. 17 and
 * Eq. 22 are piecewise constant and pass no gradient).  The mode follows the forward call:
 * patch_idx NULL (needs blk->c == blk->m, no UOE_FLAG_GATE_PATCH) = expert selection, patch_idx
 * [b,n,c] = data selection (needs blk->c < blk->m).  Given d_out = dL/d(out) [b,l,d] and the forward
 * inputs, writes, all in full and in the storage dtype unless noted:
 *   d_u     [b,l,d]     = (d_out, with UOE_FLAG_RESIDUAL) + the gradient through every active expert
 *                         (data selection: scattered back onto the tokens of its patches)
 *   d_a_in  [n,d,d_e], d_a_out [n,d_e,d]   summed over the samples that selected the expert; zero
 *                         for an expert no sample selected
 *   d_gate  [b,n] fp32  dL/d(expert_gate[b,i]) for the sample's active experts, zero elsewhere and
 *                       everywhere without UOE_FLAG_GATE_EXPERT; may be NULL
 *   d_patch_gate [b,n,m] fp32 (data selection) dL/d(patch_gate) on the selected patches of the
 *                       active experts, zero elsewhere and without UOE_FLAG_GATE_PATCH; may be NULL
 * Two paths.  bf16 storage with l, d and d_e multiples of 32, b <= 128 (and l_p a multiple of 32 in
 * data-selection mode) runs on the matrix cores, intermediates (u A^I, d_out A^O^T) kept in bf16
 * between the kernels.  Every other expert-selection request (fp32 storage, any l, d, d_e) runs on
 * the vector ALU with fp32 intermediates: general, not fast.  Data selection outside the first path
 * is UOE_ERR_UNSUPPORTED.  Outputs must not alias inputs.
 * Deterministic: fixed summation order, no atomics.  ws: at least
 * uoe_uome_backward_workspace_bytes(blk) bytes (0 = descriptor invalid or unsupported).
 */
size_t uoe_uome_backward_workspace_bytes(const uoe_block_desc *blk);
int uoe_uome_backward(const uoe_block_desc *blk, const void *u, const void *a_in, const void *a_out,
                      const int32_t *expert_idx, const float *expert_gate,
                      const int32_t *patch_idx, const float *patch_gate, const void *d_out,
                      void *d_u, void *d_a_in, void *d_a_out, float *d_gate, float *d_patch_gate,
                      void *ws, size_t ws_bytes, void *hip_stream);

typedef struct {
    const void *w_expert, *w_b, *w_a, *wq, *wk, *wv, *wo;
} uoe_smha_weights;

/*
 * Backward pass of uoe_route (the derivatives of the expert router, Eq. 21, and of the data
 * router, Eq. 13-14; the additive noise and the top-k / top-c selections pass no gradient).
 * Given the gates the forward call returned and their gradients (as the block backward calls
 * return them), writes the router weight gradients in full and ADDS the routers' share of the
 * input gradient to d_x, which is read, updated and written in place:
 *   d_w_expert [n, l*d] = dz^T vec(x),  dz = g * (dg - sum_i g_i dg_i);   d_x += dz W_E
 *   d_w_a [l,m] = sum_b (x W_B) dL,  d_w_b [d,n] = sum_b x^T (W_A dL^T),  d_x += W_A dL^T W_B^T,
 *   dL = gate * (dgate - sum over experts of gate * dgate) per patch
 * A router whose weights are NULL is skipped (its gate and gradient pointers are ignored); at
 * least one must be present; w_b and w_a come together.  Storage dtype fp32 or bf16, fp32
 * arithmetic.  Limits of this build: b <= 128, d <= 2048, (n*m + 64*n) * 4 + d*n*elem <= 64 KiB.
 * ws: at least uoe_route_backward_workspace_bytes(blk) bytes (0 = invalid or unsupported).
 */
size_t uoe_route_backward_workspace_bytes(const uoe_block_desc *blk);
int uoe_route_backward(const uoe_block_desc *blk, const void *x, const void *w_expert,
                       const void *w_b, const void *w_a, const float *expert_gate,
                       const float *patch_gate, const float *d_expert_gate,
                       const float *d_patch_gate, void *d_x, void *d_w_expert, void *d_w_b,
                       void *d_w_a, void *ws, size_t ws_bytes, void *hip_stream);

/* Gradients of the four SMHA weight tensors, shaped like the weights. */
typedef struct {
    void *d_wq, *d_wk, *d_wv, *d_wo;
} uoe_smha_weight_grads;

/*
 * Backward pass of uoe_smha_forward (the derivatives of Eq. 27-36, with the shared causal mask of
 * Sec. III-C.3 when UOE_FLAG_CAUSAL is set and the partial RoPE of Eq. 32 when rope_dim > 0; the selections of Eq. 17 and 22 are piecewise constant
 * and pass no gradient).  Given d_out = dL/d(out) [b,l,d] and the forward inputs (w->wq/wk/wv/wo;
 * the router members of w are ignored), writes, all in full:
 *   d_x [b,l,d]            (d_out, with UOE_FLAG_RESIDUAL) + the gradients scattered back from every
 *                          active expert that selected the token's patch; must not alias x or d_out
 *   dw->d_wq/d_wk/d_wv [n,d,d_h], dw->d_wo [n,d_h,d]   zero for an expert no sample selected
 *   d_expert_gate [b,n] fp32, d_patch_gate [b,n,m] fp32   dL/d(gate) for the active experts and
 *                          their selected patches, zero elsewhere and when the matching flag is
 *                          off; either may be NULL
 * pad_mask [b,l] bytes or NULL as in uoe_smha_forward_masked (Eq. 41: padded keys are out of every
 * softmax).  The forward intermediates are recomputed.  Two paths: bf16 storage with d_h in
 * {32, 64, 128}, d % 32 == 0, l_p % 32 == 0 and b <= 128 runs on the matrix cores; every other
 * request (fp32 storage, a 14-token patch, d_h = 16) runs on the vector ALU with fp32 intermediates
 * and the attention probabilities of every unit materialised ([b*k, l_a, l_a] fp32 twice in ws):
 * general, not fast, and UOE_ERR_UNSUPPORTED beyond b*k*l_a*l_a = 2^31 or c > 1024.
 * Deterministic: fixed summation order, no atomics.  ws: at least
 * uoe_smha_backward_workspace_bytes(blk) bytes (0 = descriptor invalid or unsupported).
 */
size_t uoe_smha_backward_workspace_bytes(const uoe_block_desc *blk);
int uoe_smha_backward(const uoe_block_desc *blk, const void *x, const uoe_smha_weights *w,
                      const int32_t *expert_idx, const float *expert_gate, const int32_t *patch_idx,
                      const float *patch_gate, const uint8_t *pad_mask, const void *d_out, void *d_x,
                      const uoe_smha_weight_grads *dw, float *d_expert_gate, float *d_patch_gate,
                      void *ws, size_t ws_bytes, void *hip_stream);

/* w_b [d,n] / w_a [l,m]: the UoME block's data-selection router (Eq. 13), both NULL for
 * expert selection only */
typedef struct {
    const void *w_expert, *w_b, *w_a, *a_in, *a_out;
} uoe_uome_weights;

/* Optional copies of a block's routing results; any member may be NULL. */
typedef struct {
    int32_t *expert_idx;
    float *expert_gate;
    int32_t *patch_idx;
    float *patch_gate;
} uoe_routing_out;

/*
 * One UoE layer (Sec. III-C): route on x, SMHA -> u; route on u with the UoME
 * router(s), UoME -> out.  `smha` and `uome` must agree on b, l, d and dtype.  A
 * UoME descriptor with m == c runs in expert-selection mode (the patch members of
 * `routing_m` are not written); with c < m it needs wm->w_b / wm->w_a and runs in
 * data-selection mode (no additive noise on the UoME patch logits in this call).
 * out must not alias x.
 */
int uoe_layer_forward(const uoe_block_desc *smha, const uoe_smha_weights *wa,
                      const float *noise_a_expert, const float *noise_a_patch,
                      const uoe_block_desc *uome, const uoe_uome_weights *wm,
                      const float *noise_m_expert, const void *x, void *out,
                      const uoe_routing_out *routing_a, const uoe_routing_out *routing_m, void *ws,
                      size_t ws_bytes, void *hip_stream);

/*
 * uoe_layer_forward with a padding mask on the SMHA block (Eq. 41, Sec. III-C.3): pad_mask [b,l]
 * bytes on the device, 1 = token, 0 = padding, as in uoe_smha_forward_masked (padded keys are out
 * of every attention softmax; routing and UoME see every row).  pad_mask == NULL is
 * uoe_layer_forward.  Same workspace.
 */
int uoe_layer_forward_masked(const uoe_block_desc *smha, const uoe_smha_weights *wa,
                             const float *noise_a_expert, const float *noise_a_patch,
                             const uoe_block_desc *uome, const uoe_uome_weights *wm,
                             const float *noise_m_expert, const void *x, const uint8_t *pad_mask,
                             void *out, const uoe_routing_out *routing_a,
                             const uoe_routing_out *routing_m, void *ws, size_t ws_bytes,
                             void *hip_stream);

/* Gradients of a block's router weights, shaped like the weights; a member may be NULL when the
 * block has no such router. */
typedef struct {
    void *d_w_expert, *d_w_b, *d_w_a;
} uoe_router_grads;

/*
 * Backward pass of uoe_layer_forward (Sec. III-C): the four backward calls above chained on one
 * stream.  d_out = dL/d(out) [b,l,d]  ->  uoe_uome_backward and the UoME router's
 * uoe_route_backward (on u) give dL/du  ->  uoe_smha_backward and the SMHA routers'
 * uoe_route_backward (on x) give d_x = dL/dx [b,l,d].
 *   routing_a / routing_m: the routing results of the forward call (its uoe_routing_out copies),
 *       read only; expert_idx and, for SMHA, patch_idx are required, a gate is required when its
 *       flag is set.
 *   u: the SMHA output of the forward pass, or NULL to have it recomputed from x.
 *   dwa, d_a_in, d_a_out: gradients of the block weights; dra / drm: gradients of the routers'
 *       weights (required when the block has a router; a router's gate flag must then be set,
 *       otherwise its weights have no influence on the output: UOE_ERR_INVALID_ARG).
 * Limits: those of the four calls.  A UoME block with c < m runs in data-selection mode as in the
 * forward call (wm->w_b / wm->w_a and routing_m->patch_idx required).  ws: at least
 * uoe_layer_backward_workspace_bytes(smha, uome) bytes (0 = invalid or unsupported).
 */
size_t uoe_layer_backward_workspace_bytes(const uoe_block_desc *smha, const uoe_block_desc *uome);
int uoe_layer_backward(const uoe_block_desc *smha, const uoe_smha_weights *wa,
                       const uoe_block_desc *uome, const uoe_uome_weights *wm, const void *x,
                       const void *u, const uoe_routing_out *routing_a,
                       const uoe_routing_out *routing_m, const void *d_out, void *d_x,
                       const uoe_smha_weight_grads *dwa, const uoe_router_grads *dra, void *d_a_in,
                       void *d_a_out, const uoe_router_grads *drm, void *ws, size_t ws_bytes,
                       void *hip_stream);

/*
 * Backward pass of uoe_layer_forward_masked: uoe_layer_backward with the forward call's padding
 * mask (Eq. 41) handed to the SMHA block's backward pass and to the recomputation of u.
 * pad_mask == NULL is uoe_layer_backward.  Same workspace.
 */
int uoe_layer_backward_masked(const uoe_block_desc *smha, const uoe_smha_weights *wa,
                              const uoe_block_desc *uome, const uoe_uome_weights *wm,
                              const void *x, const uint8_t *pad_mask, const void *u,
                              const uoe_routing_out *routing_a, const uoe_routing_out *routing_m,
                              const void *d_out, void *d_x, const uoe_smha_weight_grads *dwa,
                              const uoe_router_grads *dra, void *d_a_in, void *d_a_out,
                              const uoe_router_grads *drm, void *ws, size_t ws_bytes,
                              void *hip_stream);

/*
 * Measurement probes (not steps of the layer; Sec. IV-D measures run time, these give the scale to
 * read such measurements against on this GPU): what the device delivers for a plain copy, a
 * read-only stream and a register-resident bf16 MFMA loop.  A benchmark prices a kernel against the
 * published peaks and reports these beside them; the copy also calibrates hardware byte counters
 * on a transfer of known size.  All pointers are device pointers, 16-byte aligned; bytes % 16 == 0.
 *   uoe_probe_copy   dst[0..bytes) = src[0..bytes)  (reads `bytes`, writes `bytes`; no overlap)
 *   uoe_probe_read   reads src[0..bytes) and folds it into sink[0..4096) (uint32, device)
 *   uoe_probe_mfma   512 workgroups of 4 waves, each wave `iters` rounds of 8 independent
 *                    v_mfma_f32_32x32x16_bf16 on operand fragments read once from `operands`
 *                    (6 KiB, device: zeros and random values clock differently); the accumulator
 *                    sums go to sink[0..131072) (fp32, device); *flops (host, may be NULL) receives
 *                    the FLOP count of the launch
 */
int uoe_probe_copy(const void *src, void *dst, size_t bytes, void *hip_stream);
int uoe_probe_read(const void *src, size_t bytes, uint32_t *sink, void *hip_stream);
int uoe_probe_mfma(const void *operands, int32_t iters, float *sink, double *flops, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* UOE_H */

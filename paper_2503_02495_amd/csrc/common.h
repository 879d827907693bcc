// Shared device helpers and the internal launcher interface of libuoe (gfx950 only).
#pragma once
#include <cstdlib>
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace uoe {

// ---------------------------------------------------------------- storage types
struct bf16_t {
    uint16_t v;
};

// 16-byte accesses with the non-temporal hint, for bytes a call touches once: an output nobody reads
// again before the call ends, a residual at its last use.  Without the hint such streams displace, in L2
// and in the memory-side cache, the tensors that later kernels of the same call do read again
// (x, u, the hidden activations).  Operands that several workgroups share must NOT take it.
// `once` is decided on the host (stream_once): tensors that fit the caches keep the plain accesses, which
// let the next kernel find them there.
typedef unsigned int once_u32x4 __attribute__((ext_vector_type(4)));
template <bool ONCE> __device__ __forceinline__ void store16(void *p, uint4 v)
{
    const once_u32x4 w = {v.x, v.y, v.z, v.w};
    if constexpr (ONCE) __builtin_nontemporal_store(w, reinterpret_cast<once_u32x4 *>(p));
    else *reinterpret_cast<once_u32x4 *>(p) = w;
}
template <bool ONCE> __device__ __forceinline__ uint4 load16(const void *p)
{
    once_u32x4 w;
    if constexpr (ONCE) w = __builtin_nontemporal_load(reinterpret_cast<const once_u32x4 *>(p));
    else w = *reinterpret_cast<const once_u32x4 *>(p);
    return make_uint4(w.x, w.y, w.z, w.w);
}
// a tensor of this many bytes is streamed past the caches (measured: 67 MB and up gain, 34 MB and down lose);
// UOE_STREAM_ONCE_MIN_BYTES in the environment overrides the threshold (0: always, for tests of the hinted paths)
inline bool stream_once(size_t bytes)
{
    const char *env = getenv("UOE_STREAM_ONCE_MIN_BYTES");
    const double min_bytes = env ? atof(env) : 48.0 * 1048576.0;
    return (double)bytes >= min_bytes;
}

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return __uint_as_float(((uint32_t)x.v) << 16); }

// round to nearest, ties to even (inputs are finite by contract)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <typename T> __device__ __forceinline__ T from_f32(float f);
template <> __device__ __forceinline__ float from_f32<float>(float f) { return f; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float f)
{
    bf16_t r;
    r.v = f32_to_bf16_bits(f);
    return r;
}

// 8 consecutive elements (16-byte aligned for bf16, 32-byte span for fp32) -> fp32
__device__ __forceinline__ void load8(const float *p, float (&o)[8])
{
    const float4 a = *reinterpret_cast<const float4 *>(p);
    const float4 b = *reinterpret_cast<const float4 *>(p + 4);
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
    o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16_t *p, float (&o)[8])
{
    const uint4 a = *reinterpret_cast<const uint4 *>(p);
    o[0] = __uint_as_float(a.x << 16); o[1] = __uint_as_float(a.x & 0xFFFF0000u);
    o[2] = __uint_as_float(a.y << 16); o[3] = __uint_as_float(a.y & 0xFFFF0000u);
    o[4] = __uint_as_float(a.z << 16); o[5] = __uint_as_float(a.z & 0xFFFF0000u);
    o[6] = __uint_as_float(a.w << 16); o[7] = __uint_as_float(a.w & 0xFFFF0000u);
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Routing indices are caller data: clamp them into [0, count) so that a corrupt index can read the
// wrong row but never leave the tensor.
__device__ __forceinline__ int clampi(int v, int count) { return min(max(v, 0), count - 1); }

__device__ __forceinline__ float silu(float z) { return z / (1.0f + __expf(-z)); }
// SiLU with the hardware exp2 and reciprocal (about 1 ulp each): for epilogues that round the
// result to bf16 anyway
__device__ __forceinline__ float silu_fast(float z)
{
    return z * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * z));
}

// ---------------------------------------------------------------- flags (mirror of the ABI values)
constexpr uint32_t F_RESIDUAL = 1u, F_GATE_EXPERT = 2u, F_GATE_PATCH = 4u, F_CAUSAL = 8u;

// ---------------------------------------------------------------- launcher arguments
struct RouteArgs {
    const void *x, *w_e, *w_b, *w_a;          // w_e NULL: no expert router; w_b NULL: no data router
    const float *noise_e, *noise_p;
    int b, l, d, n, k, m, c;
    int tc, nchunks;                          // expert router: tokens per chunk, chunks per sample
    int tc_d, nchunks_d;                      // data router: the same
    float *zpart, *gpart;                     // [nchunks, b, n], [nchunks_d, b, n*m]
    float *gred;                              // [b, n*m]
    float *t1;                                // [b, l, n]: per-token expert scores x W_B of the one-pass kernel
    int32_t *expert_idx, *patch_idx;          // outputs (any may be NULL)
    float *expert_gate, *patch_gate;
    // dynamic capacity (Eq. 15-16) and balance statistics (Eq. 43-44): capacity NULL = not asked for
    int patch_k;                              // experts each patch names in stage 1
    int32_t *capacity;                        // [b]
    float *load_f, *load_p;                   // [b,n] each, or NULL
};

struct SmhaArgs {
    const void *x, *wq, *wk, *wv, *wo;
    const int32_t *expert_idx, *patch_idx;
    const float *expert_gate, *patch_gate;    // NULL when the matching flag is off
    void *out;
    int b, l, d, n, k, m, c, d_h;
    uint32_t flags;
    int rope_dim;                             // rotary dims at the end of a head (Eq. 32), 0 = none
    const unsigned char *pad_mask;            // [b,l] 1 = token, 0 = padding (Eq. 41), or NULL
    // workspace
    void *q, *kk, *v, *o, *o_lo;              // [b*k, l_a, d_h] each, storage dtype (o_lo: low part of o, MFMA path)
    int32_t *inv_cnt, *inv_ent;               // [b,m], [b,m,k]: which (slot s, pick t) chose patch p
    float *lse;                               // [b*k, l_a] or NULL: base-2 log-sum-exp of each query's scaled logits
                                              // (MFMA attention only; kept for the backward pass)
    int keep_v_bf16;                          // 1: the MFMA path leaves v in bf16 (the backward pass reads it); 0: it
                                              // writes v as fp16, the operand format of the attention kernel's P V
    uint32_t skip;                            // steps NOT to run (SMHA_STEP_* bits; 0 = the whole block): a caller
                                              // that times one step runs it on what the others left in the workspace
};
constexpr uint32_t SMHA_STEP_QKV = 1u, SMHA_STEP_ATTENTION = 2u, SMHA_STEP_OUT = 4u;

struct UomeArgs {
    const void *u, *a_in, *a_out;
    const int32_t *expert_idx;
    const float *expert_gate;                 // NULL when GATE_EXPERT is off
    void *out;
    int b, l, d, n, k, d_e;
    uint32_t flags;
    void *hidden;                             // [b, l, k*d_e], storage dtype
};

// UoME with patch-wise data selection (Eq. 37-40): routing as for SMHA, hidden per active unit
struct UomeDsArgs {
    const void *u, *a_in, *a_out;
    const int32_t *expert_idx, *patch_idx;
    const float *expert_gate, *patch_gate;    // NULL when the matching flag is off
    void *out;
    int b, l, d, n, k, m, c, d_e;
    uint32_t flags;
    void *hidden;                             // [b*k, l_a, d_e], storage dtype
    int32_t *inv_cnt, *inv_ent;               // [b,m], [b,m,k] (engines without in-kernel segment lists)
};

// Backward pass of the expert-selection UoME block (bf16 storage, MFMA shapes only)
struct UomeBwdArgs {
    const void *u, *a_in, *a_out, *d_out;
    const int32_t *expert_idx;
    const float *expert_gate;                 // NULL when GATE_EXPERT is off
    void *d_u, *d_a_in, *d_a_out;             // [b,l,d], [n,d,d_e], [n,d_e,d], storage dtype
    float *d_gate;                            // [b,n] or NULL
    int b, l, d, n, k, d_e;
    uint32_t flags;
    // workspace, storage dtype unless noted
    void *z, *dh, *dz;                        // [b, l, k*d_e] each
    void *dz_t, *h_t;                         // [b, k*d_e, l] each
    void *a_in_t, *a_out_t;                   // [n, d_e, d], [n, d, d_e]
    float *gpart;                             // [b, k, gchunks] partial sums of d_gate
    float *partial;                           // [2*n*splits, d_e, d] split-K tiles of the two weight gradients
    int gchunks, splits;
    // data-selection mode (patch_idx != NULL): units = (sample, slot) with l_a = c*l/m gathered rows;
    // z, dh, dz are [units, l_a, d_e], dz_t and h_t [units, d_e, l_a]
    const int32_t *patch_idx;
    const float *patch_gate;                  // NULL when GATE_PATCH is off
    float *d_patch_gate;                      // [b,n,m] or NULL
    float *rt;                                // [units, l_a]: dL/d(weight of row t)
    int m, c;
};

// Backward pass of the SMHA block
struct SmhaBwdArgs {
    SmhaArgs f;                               // the forward call that is recomputed: no gates in f.flags, f.lse set
    const void *d_out;                        // [b,l,d]
    const float *expert_gate, *patch_gate;    // as in the forward call (NULL when the flag is off)
    uint32_t flags;                           // the block's flags
    void *d_x, *d_wq, *d_wk, *d_wv, *d_wo;    // [b,l,d], 3 x [n,d,d_h], [n,d_h,d], storage dtype
    float *d_expert_gate, *d_patch_gate;      // [b,n], [b,n,m], or NULL
    // workspace, storage dtype unless noted
    void *wo_t, *wqkv_t;                      // [n, d, d_h], [n, 3*d_h, d]
    float *do_raw;                            // [units, l_a, d_h] fp32
    void *d_o;                                // [units, l_a, d_h]
    void *o_t;                                // [units, d_h, l_a]
    void *dqkv, *dqkv_t;                      // [units, l_a, 3*d_h], [units, 3*d_h, l_a]
    float *rt, *dd;                           // [units, l_a] each: dL/dw_t and the softmax row term
    float *partial;                           // [4*n*splits, d_h, d] split tiles of the four weight gradients
    int splits;
    // vector-ALU path only (any shape, any storage type): every workspace array above that it uses is fp32
    float *probs, *dscores;                   // [units, l_a, l_a] each: softmax probabilities and score gradients
    float *wt;                                // transposed fp32 copies of the weights: W^{q,k,v} as [3][n][d_h][d], then W^O as [n][d][d_h]
};

// Backward pass of the routers of one block
struct RouteBwdArgs {
    const void *x, *w_e, *w_b, *w_a;          // w_e NULL: no expert router; w_b NULL: no data router
    const float *g_e, *g_p;                   // gates of the forward pass [b,n], [b,n,m]
    const float *d_g_e, *d_g_p;               // their gradients
    void *d_x;                                // [b,l,d] in/out: the routers' contribution is added
    void *d_w_e, *d_w_b, *d_w_a;              // [n,l*d], [d,n], [l,m], storage dtype
    int b, l, d, n, m;
    // workspace (fp32)
    float *dz, *dl;                           // [b,n], [b,n,m]: gradients of the router logits
    float *t1, *u;                            // [b,l,n] each: x W_B and W_A dL^T
    float *wb_part;                           // [wb_chunks, d, n] partial sums of dW_B
    int wb_tokens, wb_chunks;                 // tokens per chunk, chunks over the b*l tokens
};

struct GatherArgs {
    const void *x;
    const int32_t *expert_idx, *patch_idx;
    void *h;
    int b, l, d, n, k, m, c;
};

// Launchers: enqueue on `st`, return the runtime's launch status.
hipError_t launch_route(const RouteArgs &a, bool bf16, hipStream_t st);
hipError_t launch_balance_loss(const float *load_f, const float *load_p, float alpha, float *loss, float *d_patch_gate,
                               int b, int n, int m, hipStream_t st);
hipError_t launch_gather(const GatherArgs &a, bool bf16, hipStream_t st);
hipError_t launch_smha(const SmhaArgs &a, bool bf16, hipStream_t st);
// Eq. 28-34 of the MFMA path only (projections, rotary embedding, attention into a.o / a.o_lo / a.lse);
// the caller has checked bf16 storage, d % 32 == 0 and d_h in {32, 64, 128}
hipError_t launch_smha_qkv_attention(const SmhaArgs &a, hipStream_t st);
hipError_t launch_uome(const UomeArgs &a, bool bf16, hipStream_t st);
hipError_t launch_uome_up(const UomeArgs &a, bool bf16, hipStream_t st);    // Eq. 38 only
hipError_t launch_uome_down(const UomeArgs &a, bool bf16, hipStream_t st);  // Eq. 39-40 only
hipError_t launch_uome_ds(const UomeDsArgs &a, bool bf16, hipStream_t st);
hipError_t launch_uome_backward(const UomeBwdArgs &a, hipStream_t st);
hipError_t launch_smha_backward(const SmhaBwdArgs &a, hipStream_t st);
// gate gradients of the units of a data-selected block from the row terms a.rt (uses the routing
// fields of a.f, a.flags, the gates and the two outputs, which it clears first)
hipError_t launch_unit_gate_grads(const SmhaBwdArgs &a, hipStream_t st);
// vector-ALU backward passes for the shapes and storage types the matrix-core kernels do not take
hipError_t launch_uome_backward_generic(const UomeBwdArgs &a, bool bf16, hipStream_t st);
hipError_t launch_smha_backward_generic(const SmhaBwdArgs &a, bool bf16, hipStream_t st);
hipError_t launch_route_backward(const RouteBwdArgs &a, bool bf16, hipStream_t st);
int smha_backward_splits(int b, int n, int k, int c);
int uome_backward_gate_chunks(int l, int d_e);
int uome_backward_splits(int b, int l, int d, int n, int k, int d_e);

// measurement probes (probe.hip)
constexpr unsigned PROBE_READ_BLOCKS = 256 * 16, PROBE_MFMA_BLOCKS = 256 * 2;
hipError_t launch_probe_copy(const void *src, void *dst, size_t bytes, hipStream_t st);
hipError_t launch_probe_read(const void *src, size_t bytes, uint32_t *sink, hipStream_t st);
hipError_t launch_probe_mfma(const void *operands, int iters, float *sink, hipStream_t st);

// host-side sizing shared by api.cpp and the launchers
int route_tokens_per_chunk(int b, int l);
int route_expert_mfma_tokens_per_chunk(int b, int l, int d, int n);
int route_data_tokens_per_chunk(int b, int l, int d, int n, bool bf16);
// streaming router kernel: applicability and launch shape (host side)
constexpr int ROUTE_STREAM_CHUNKS = 256;      // one workgroup per compute unit
struct RouteStreamPlan {
    bool ok;             // the kernel applies to this shape
    int rt, ct, rb;      // 16-sample tiles per workgroup, 16-expert tiles, bytes per row per stage
    int tpc, nchunks;    // tokens per chunk, chunks
    int ipw;             // load instructions per wave per stage
    size_t lds;          // dynamic LDS bytes
};
RouteStreamPlan route_stream_plan(int b, int l, int d, int n, bool bf16, bool has_d);
struct RouteFoldPlan {
    int tr, ranges;      // tokens per range, ranges per sample
};
RouteFoldPlan route_fold_plan(int b, int l);

}  // namespace uoe

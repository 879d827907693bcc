// C ABI of libuoe: host-side argument validation, workspace carving and kernel dispatch.
// Nothing here allocates or synchronises; every entry point validates, then enqueues.
#include "../../include/uoe.h"
#include "common.h"
#include <mutex>

using namespace uoe;

// Scratch of uoe_route_static, the entry point that allocates nothing: a fixed array in device
// memory, one copy per GPU the library runs on, held until the process ends.  In host code this
// name is only a handle for hipGetSymbolAddress; kernels get the address that call returns.
static __device__ __align__(256) unsigned char scratch[UOE_ROUTE_STATIC_SCRATCH_BYTES];

namespace {

constexpr size_t ALIGN = 256;
inline size_t up(size_t v) { return (v + ALIGN - 1) & ~(ALIGN - 1); }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t elem_size(int dtype) { return dtype == UOE_BF16 ? 2 : 4; }

// Generic descriptor checks shared by every call.  kind: what the descriptor is used for.
enum DescKind { DESC_ROUTE, DESC_SMHA, DESC_UOME };
int check_desc(const uoe_block_desc *d, DescKind kind)
{
    const bool smha = kind == DESC_SMHA;
    if (!d) return UOE_ERR_INVALID_ARG;
    if (d->b < 1 || d->l < 1 || d->d < 1 || d->n < 1 || d->k < 1 || d->k > d->n || d->m < 1 ||
        d->c < 1 || d->c > d->m || d->width < 1 || (d->l % d->m) != 0)
        return UOE_ERR_INVALID_ARG;
    if (d->dtype != UOE_F32 && d->dtype != UOE_BF16) return UOE_ERR_INVALID_ARG;
    if (d->flags & ~(uint32_t)(UOE_FLAG_RESIDUAL | UOE_FLAG_GATE_EXPERT | UOE_FLAG_GATE_PATCH | UOE_FLAG_CAUSAL))
        return UOE_ERR_INVALID_ARG;
    for (int i = 0; i < 5; ++i)
        if (d->reserved[i] != 0) return UOE_ERR_INVALID_ARG;
    if (d->rope_dim < 0 || (d->rope_dim & 1) || d->rope_dim > d->width) return UOE_ERR_INVALID_ARG;
    // the causal mask and RoPE belong to the attention block (routing and gathering ignore them)
    if (kind == DESC_UOME && (d->rope_dim != 0 || (d->flags & UOE_FLAG_CAUSAL))) return UOE_ERR_UNSUPPORTED;
    if (d->n > 32 || (d->d % 8) != 0 || (d->width % 8) != 0 || d->m > 1024) return UOE_ERR_UNSUPPORTED;
    if ((long)d->n * d->m > 8192) return UOE_ERR_UNSUPPORTED;
    if ((long)d->b * d->m > 65535 || (long)d->b * d->k > 65535) return UOE_ERR_UNSUPPORTED;
    const long wide = (long)d->k * d->width > d->d ? (long)d->k * d->width : d->d;
    if ((double)d->b * d->l * (double)wide > 1.0e12) return UOE_ERR_UNSUPPORTED;  // keeps all index math in range
    if (smha && d->width > 128) return UOE_ERR_UNSUPPORTED;
    return UOE_OK;
}

struct RouteWs {
    int tc, nchunks, tc_d, nchunks_d;
    size_t zpart, gpart, gred, t1, total;
};
RouteWs route_ws(int b, int l, int d, int n, int m, bool bf16)
{
    RouteWs w;
    w.tc = bf16 ? route_expert_mfma_tokens_per_chunk(b, l, d, n) : route_tokens_per_chunk(b, l);
    w.nchunks = (l + w.tc - 1) / w.tc;
    w.tc_d = route_data_tokens_per_chunk(b, l, d, n, bf16);
    w.nchunks_d = (l + w.tc_d - 1) / w.tc_d;
    size_t off = 0;
    w.zpart = off; off += up((size_t)w.nchunks * b * n * sizeof(float));
    w.gpart = off; off += up((size_t)w.nchunks_d * b * n * m * sizeof(float));
    w.gred = off;  off += up((size_t)b * n * m * sizeof(float));
    w.t1 = off;    off += route_stream_plan(b, l, d, n, bf16, true).ok ? up((size_t)b * l * n * sizeof(float)) : 0;
    w.total = off;
    return w;
}

struct SmhaWs {
    size_t q, k, v, o, o_lo, inv_cnt, inv_ent, total;
};
SmhaWs smha_ws(const uoe_block_desc *d)
{
    SmhaWs w;
    const size_t l_a = (((size_t)d->c * (d->l / d->m)) + 7) & ~(size_t)7;  // v may be stored transposed, rows padded to 8
    const size_t one = up((size_t)d->b * d->k * l_a * d->width * elem_size(d->dtype));
    size_t off = 0;
    w.q = off; off += one;
    w.k = off; off += one;
    w.v = off; off += one;
    w.o = off; off += one;
    w.o_lo = off; off += one;
    w.inv_cnt = off; off += up((size_t)d->b * d->m * sizeof(int32_t));
    w.inv_ent = off; off += up((size_t)d->b * d->m * d->k * sizeof(int32_t));
    w.total = off;
    return w;
}

// hidden activations: [b, l, k*d_e] (expert selection) or [b*k, l_a, d_e] (data selection, never
// larger); behind them the inverse map of the data-selection mode
struct UomeWs {
    size_t hidden, inv_cnt, inv_ent, total;
};
UomeWs uome_ws_layout(const uoe_block_desc *d)
{
    UomeWs w;
    size_t off = 0;
    w.hidden = off; off += up((size_t)d->b * d->l * d->k * d->width * elem_size(d->dtype));
    w.inv_cnt = off; off += up((size_t)d->b * d->m * sizeof(int32_t));
    w.inv_ent = off; off += up((size_t)d->b * d->m * d->k * sizeof(int32_t));
    w.total = off;
    return w;
}
size_t uome_ws(const uoe_block_desc *d) { return uome_ws_layout(d).total; }

// backward pass of the UoME block: Z, dH, dZ [b,l,k*d_e]; dZ^T, H^T [b,k*d_e,l]; the two transposed
// weight tensors; split-K tiles of one weight gradient; partial sums of the gate gradient
struct UomeBwdWs {
    size_t z, dh, dz, dz_t, h_t, a_in_t, a_out_t, partial, gpart, rt, total;
    int splits;
};
static bool uome_bwd_mfma(const uoe_block_desc *blk);
UomeBwdWs uome_bwd_ws(const uoe_block_desc *d)
{
    UomeBwdWs w{};
    if (!uome_bwd_mfma(d)) {  // vector-ALU path: Z/H and dH/dZ in fp32
        const size_t act32 = up((size_t)d->b * d->l * d->k * d->width * sizeof(float));
        w.z = 0; w.dh = act32; w.total = 2 * act32;
        // weight gradients: the (sample, slot) pairs cut into ranges (at most 8) until about 4096 tiles of
        // 64x64 exist, a few rounds of them per CU; partial tiles in fp32, added in range order
        const long tiles = 2L * d->n * ((d->d + 63) / 64) * ((d->width + 63) / 64);
        long s = 4096 / tiles;
        s = s < 1 ? 1 : (s > 8 ? 8 : s);
        if (s > (long)d->b * d->k) s = (long)d->b * d->k;
        w.splits = (int)s;
        if (w.splits > 1) {
            w.partial = w.total;
            w.total += up((size_t)2 * d->n * w.splits * d->d * d->width * sizeof(float));
        }
        return w;
    }
    const size_t es = elem_size(d->dtype);
    const size_t act = up((size_t)d->b * d->l * d->k * d->width * es);
    const size_t wt = up((size_t)d->n * d->d * d->width * es);
    size_t off = 0;
    w.z = off; off += act;
    w.dh = off; off += act;
    w.dz = off; off += act;
    w.dz_t = off; off += act;
    w.h_t = off; off += act;
    w.a_in_t = off; off += wt;
    w.a_out_t = off; off += wt;
    // data-selection mode (c < m) works on at most as many rows (units * l_a <= b * k * l) in the same
    // buffers; its weight gradients are cut by (unit, pick) segments instead of token ranges
    w.splits = d->c < d->m ? smha_backward_splits(d->b, d->n, d->k, d->c)
                           : uome_backward_splits(d->b, d->l, d->d, d->n, d->k, d->width);
    w.partial = off;
    off += up(2 * (size_t)d->n * w.splits * d->d * d->width * sizeof(float));  // both weight gradients
    w.gpart = off; off += up((size_t)d->b * d->k * uome_backward_gate_chunks(d->l, d->width) * sizeof(float));
    w.rt = off; off += up((size_t)d->b * d->k * d->l * sizeof(float));
    w.total = off;
    return w;
}
// the matrix-core backward takes bf16 storage and 32-multiples; everything else goes to the vector-ALU path
static bool uome_bwd_mfma(const uoe_block_desc *blk)
{
    if (blk->dtype != UOE_BF16) return false;
    if (blk->l % 32 || blk->d % 32 || blk->width % 32 || blk->b > 128) return false;
    if (blk->c < blk->m && (blk->l / blk->m) % 32) return false;
    return true;
}
int check_uome_bwd(const uoe_block_desc *blk)
{
    const int rc = check_desc(blk, DESC_UOME);
    if (rc != UOE_OK) return rc;
    // the vector-ALU path covers the expert-selection mode only
    if (!uome_bwd_mfma(blk) && blk->c < blk->m) return UOE_ERR_UNSUPPORTED;
    return UOE_OK;
}

// backward pass of the SMHA block: the forward's scratch, then the backward's own
struct SmhaBwdWs {
    SmhaWs fwd;
    size_t lse, rt, dd, wo_t, wqkv_t, do_raw, d_o, o_t, dqkv, dqkv_t, partial, total;
    size_t g_q, g_k, g_v, g_o, g_probs, g_dscores, g_wt;  // vector-ALU path (fp32 arrays)
    int g_splits;                                           // vector-ALU path: unit ranges of the weight gradients
};
static bool smha_bwd_mfma(const uoe_block_desc *blk)
{
    if (blk->dtype != UOE_BF16) return false;
    if (blk->width != 32 && blk->width != 64 && blk->width != 128) return false;
    return !(blk->d % 32 || (blk->l / blk->m) % 32 || blk->b > 128);
}
SmhaBwdWs smha_bwd_ws(const uoe_block_desc *d)
{
    SmhaBwdWs w{};
    if (!smha_bwd_mfma(d)) {
        const size_t l_a = (size_t)d->c * (d->l / d->m), units = (size_t)d->b * d->k;
        const size_t rows = up(units * l_a * sizeof(float)), one = up(units * l_a * d->width * sizeof(float));
        const size_t sq = up(units * l_a * l_a * sizeof(float));
        size_t off = 0;
        w.g_q = off; off += one;
        w.g_k = off; off += one;
        w.g_v = off; off += one;
        w.g_o = off; off += one;
        w.do_raw = off; off += one;
        w.dqkv = off; off += 3 * one;
        w.rt = off; off += rows;
        w.g_probs = off; off += sq;
        w.g_dscores = off; off += sq;
        w.g_wt = off; off += up((size_t)4 * d->n * d->d * d->width * sizeof(float));
        // weight gradients: the units cut into ranges until about 16 waves per SIMD are in flight, partial
        // sums in fp32, added in range order
        const size_t per = (size_t)d->n * d->d * d->width;
        size_t sp = (16384 * 64 + per - 1) / per;
        sp = sp < 1 ? 1 : (sp > 8 ? 8 : sp);
        if (sp > units) sp = units;
        w.g_splits = (int)sp;
        w.partial = off;
        if (sp > 1) off += up(sp * 4 * per * sizeof(float));
        w.total = off;
        return w;
    }
    w.fwd = smha_ws(d);
    const size_t es = elem_size(d->dtype);
    const size_t l_a = (size_t)d->c * (d->l / d->m), units = (size_t)d->b * d->k;
    const size_t rows = up(units * l_a * sizeof(float)), one = up(units * l_a * d->width * es);
    size_t off = w.fwd.total;
    w.lse = off; off += rows;
    w.rt = off; off += rows;
    w.dd = off; off += rows;
    w.wo_t = off; off += up((size_t)d->n * d->d * d->width * es);
    w.wqkv_t = off; off += up(3 * (size_t)d->n * d->d * d->width * es);
    w.do_raw = off; off += up(units * l_a * d->width * sizeof(float));
    w.d_o = off; off += one;
    w.o_t = off; off += one;
    w.dqkv = off; off += 3 * one;
    w.dqkv_t = off; off += 3 * one;
    w.partial = off;
    off += up((size_t)d->n * smha_backward_splits(d->b, d->n, d->k, d->c) * 4 * d->width * d->d * sizeof(float));
    w.total = off;
    return w;
}
int check_smha_bwd(const uoe_block_desc *blk)
{
    const int rc = check_desc(blk, DESC_SMHA);
    if (rc != UOE_OK) return rc;
    if (!smha_bwd_mfma(blk)) {
        // vector-ALU path: the materialised [units, l_a, l_a] arrays bound the size; the gate kernel holds c sums
        const size_t l_a = (size_t)blk->c * (blk->l / blk->m);
        if (blk->c > 1024 || (size_t)blk->b * blk->k * l_a * l_a > ((size_t)1 << 31)) return UOE_ERR_UNSUPPORTED;
    }
    return UOE_OK;
}

// backward pass of the routers
struct RouteBwdWs {
    size_t dz, dl, t1, u, wb_part, total;
    int wb_tokens, wb_chunks;
};
RouteBwdWs route_bwd_ws(const uoe_block_desc *d)
{
    RouteBwdWs w;
    // chunks of the token axis for dW_B: about 512 of them, 32 to 128 tokens each (the kernel stages a
    // chunk's rows of U in LDS)
    const size_t tokens = (size_t)d->b * d->l;
    w.wb_tokens = (int)((tokens + 511) / 512);
    w.wb_tokens = w.wb_tokens < 32 ? 32 : (w.wb_tokens > 128 ? 128 : w.wb_tokens);
    w.wb_chunks = (int)((tokens + w.wb_tokens - 1) / w.wb_tokens);
    size_t off = 0;
    w.dz = off; off += up((size_t)d->b * d->n * sizeof(float));
    w.dl = off; off += up((size_t)d->b * d->n * d->m * sizeof(float));
    w.t1 = off; off += up((size_t)d->b * d->l * d->n * sizeof(float));
    w.u = off; off += up((size_t)d->b * d->l * d->n * sizeof(float));
    w.wb_part = off; off += up((size_t)w.wb_chunks * d->d * d->n * sizeof(float));
    w.total = off;
    return w;
}
int check_route_bwd(const uoe_block_desc *blk)
{
    const int rc = check_desc(blk, DESC_ROUTE);
    if (rc != UOE_OK) return rc;
    if (blk->b > 128 || blk->d > 2048) return UOE_ERR_UNSUPPORTED;
    // the data router's per-token kernel stages dL [n,m], U [64,n] and W_B [d,n] in LDS
    const size_t lds = ((size_t)blk->n * blk->m + 64 * (size_t)blk->n) * sizeof(float) + 16 + (size_t)blk->d * blk->n * elem_size(blk->dtype);
    if (lds > 64 * 1024) return UOE_ERR_UNSUPPORTED;
    return UOE_OK;
}

struct RoutingBuf {
    size_t expert_idx, expert_gate, patch_idx, patch_gate, total;
};
RoutingBuf routing_buf(const uoe_block_desc *d, int m, int c)
{
    RoutingBuf r;
    size_t off = 0;
    r.expert_idx = off;  off += up((size_t)d->b * d->k * sizeof(int32_t));
    r.expert_gate = off; off += up((size_t)d->b * d->n * sizeof(float));
    r.patch_idx = off;   off += up((size_t)d->b * d->n * c * sizeof(int32_t));
    r.patch_gate = off;  off += up((size_t)d->b * d->n * m * sizeof(float));
    r.total = off;
    return r;
}

inline char *at(void *ws, size_t off) { return static_cast<char *>(ws) + off; }

// Device address of `scratch` on the current device, looked up once per device.
constexpr int MAX_DEVICES = 64;
std::mutex scratch_mutex;
void *scratch_ptr[MAX_DEVICES] = {};
int static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return UOE_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return UOE_ERR_DEVICE;
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return UOE_OK;
}

// validated routing launch; `m`/`c` are passed separately so a UoME block routes with m = c = 1
int do_route(const uoe_block_desc *blk, int m, int c, const void *x, const void *w_expert, const void *w_b,
             const void *w_a, const float *noise_expert, const float *noise_patch, int32_t *expert_idx,
             float *expert_gate, int32_t *patch_idx, float *patch_gate, void *ws, size_t ws_bytes,
             hipStream_t st)
{
    if (!x || !aligned16(x) || !aligned16(w_expert) || !aligned16(w_b) || !aligned16(w_a))
        return UOE_ERR_INVALID_ARG;
    if ((w_b == nullptr) != (w_a == nullptr)) return UOE_ERR_INVALID_ARG;
    if (!w_expert && blk->k != blk->n) return UOE_ERR_INVALID_ARG;
    if (!w_b && c != m) return UOE_ERR_INVALID_ARG;
    if ((!w_expert && noise_expert) || (!w_b && noise_patch)) return UOE_ERR_INVALID_ARG;
    // the data router stages W_B (n*d elements) in LDS
    if (w_b && (size_t)blk->n * blk->d * elem_size(blk->dtype) > 48 * 1024) return UOE_ERR_UNSUPPORTED;
    const RouteWs w = route_ws(blk->b, blk->l, blk->d, blk->n, m, blk->dtype == UOE_BF16);
    if (!ws || ws_bytes < w.total || !aligned16(ws)) return UOE_ERR_WORKSPACE;

    RouteArgs a{};
    a.x = x; a.w_e = w_expert; a.w_b = w_b; a.w_a = w_a;
    a.noise_e = noise_expert; a.noise_p = noise_patch;
    a.b = blk->b; a.l = blk->l; a.d = blk->d; a.n = blk->n; a.k = blk->k; a.m = m; a.c = c;
    a.tc = w.tc; a.nchunks = w.nchunks; a.tc_d = w.tc_d; a.nchunks_d = w.nchunks_d;
    a.zpart = reinterpret_cast<float *>(at(ws, w.zpart));
    a.gpart = reinterpret_cast<float *>(at(ws, w.gpart));
    a.gred = reinterpret_cast<float *>(at(ws, w.gred));
    a.t1 = reinterpret_cast<float *>(at(ws, w.t1));
    a.expert_idx = expert_idx; a.patch_idx = patch_idx;
    a.expert_gate = expert_gate; a.patch_gate = patch_gate;
    return launch_route(a, blk->dtype == UOE_BF16, st) == hipSuccess ? UOE_OK : UOE_ERR_DEVICE;
}

int do_smha(const uoe_block_desc *blk, const void *x, const void *wq, const void *wk, const void *wv,
            const void *wo, const int32_t *expert_idx, const float *expert_gate, const int32_t *patch_idx,
            const float *patch_gate, const uint8_t *pad_mask, void *out, void *ws, size_t ws_bytes, hipStream_t st,
            uint32_t skip = 0)
{
    if (!x || !wq || !wk || !wv || !wo || !expert_idx || !patch_idx || !out) return UOE_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(wq) || !aligned16(wk) || !aligned16(wv) || !aligned16(wo) || !aligned16(out))
        return UOE_ERR_INVALID_ARG;
    if (out == x) return UOE_ERR_INVALID_ARG;
    if ((blk->flags & UOE_FLAG_GATE_EXPERT) && !expert_gate) return UOE_ERR_INVALID_ARG;
    if ((blk->flags & UOE_FLAG_GATE_PATCH) && !patch_gate) return UOE_ERR_INVALID_ARG;
    const SmhaWs w = smha_ws(blk);
    if (!ws || ws_bytes < w.total || !aligned16(ws)) return UOE_ERR_WORKSPACE;

    SmhaArgs a{};
    a.x = x; a.wq = wq; a.wk = wk; a.wv = wv; a.wo = wo;
    a.expert_idx = expert_idx; a.patch_idx = patch_idx;
    a.expert_gate = expert_gate; a.patch_gate = patch_gate;
    a.out = out;
    a.b = blk->b; a.l = blk->l; a.d = blk->d; a.n = blk->n; a.k = blk->k; a.m = blk->m; a.c = blk->c;
    a.d_h = blk->width; a.flags = blk->flags;
    a.rope_dim = blk->rope_dim; a.pad_mask = pad_mask; a.skip = skip;
    a.q = at(ws, w.q); a.kk = at(ws, w.k); a.v = at(ws, w.v); a.o = at(ws, w.o); a.o_lo = at(ws, w.o_lo);
    a.inv_cnt = reinterpret_cast<int32_t *>(at(ws, w.inv_cnt));
    a.inv_ent = reinterpret_cast<int32_t *>(at(ws, w.inv_ent));
    return launch_smha(a, blk->dtype == UOE_BF16, st) == hipSuccess ? UOE_OK : UOE_ERR_DEVICE;
}

// patch_idx NULL: expert-selection mode (needs c == m and no patch gate).  Otherwise the
// data-selection mode of Eq. 37: every active expert processes its c selected patches.
int do_uome(const uoe_block_desc *blk, const void *u, const void *a_in, const void *a_out,
            const int32_t *expert_idx, const float *expert_gate, const int32_t *patch_idx,
            const float *patch_gate, void *out, void *ws, size_t ws_bytes, hipStream_t st)
{
    if (!u || !a_in || !a_out || !expert_idx || !out) return UOE_ERR_INVALID_ARG;
    if (!aligned16(u) || !aligned16(a_in) || !aligned16(a_out) || !aligned16(out)) return UOE_ERR_INVALID_ARG;
    if (out == u) return UOE_ERR_INVALID_ARG;
    if ((blk->flags & UOE_FLAG_GATE_EXPERT) && !expert_gate) return UOE_ERR_INVALID_ARG;
    if (!patch_idx && (blk->c != blk->m || (blk->flags & UOE_FLAG_GATE_PATCH))) return UOE_ERR_INVALID_ARG;
    if ((blk->flags & UOE_FLAG_GATE_PATCH) && !patch_gate) return UOE_ERR_INVALID_ARG;
    if (!ws || ws_bytes < uome_ws(blk) || !aligned16(ws)) return UOE_ERR_WORKSPACE;
    if (patch_idx) {
        const UomeWs w = uome_ws_layout(blk);
        UomeDsArgs a{};
        a.u = u; a.a_in = a_in; a.a_out = a_out;
        a.expert_idx = expert_idx; a.patch_idx = patch_idx;
        a.expert_gate = expert_gate; a.patch_gate = patch_gate;
        a.out = out;
        a.b = blk->b; a.l = blk->l; a.d = blk->d; a.n = blk->n; a.k = blk->k; a.m = blk->m; a.c = blk->c;
        a.d_e = blk->width;
        a.flags = blk->flags;
        a.hidden = at(ws, w.hidden);
        a.inv_cnt = reinterpret_cast<int32_t *>(at(ws, w.inv_cnt));
        a.inv_ent = reinterpret_cast<int32_t *>(at(ws, w.inv_ent));
        return launch_uome_ds(a, blk->dtype == UOE_BF16, st) == hipSuccess ? UOE_OK : UOE_ERR_DEVICE;
    }

    UomeArgs a{};
    a.u = u; a.a_in = a_in; a.a_out = a_out;
    a.expert_idx = expert_idx; a.expert_gate = expert_gate;
    a.out = out;
    a.b = blk->b; a.l = blk->l; a.d = blk->d; a.n = blk->n; a.k = blk->k; a.d_e = blk->width;
    a.flags = blk->flags;
    a.hidden = ws;
    return launch_uome(a, blk->dtype == UOE_BF16, st) == hipSuccess ? UOE_OK : UOE_ERR_DEVICE;
}

}  // namespace

extern "C" {

const char *uoe_status_string(int status)
{
    switch (status) {
        case UOE_OK: return "ok";
        case UOE_ERR_INVALID_ARG: return "invalid argument";
        case UOE_ERR_UNSUPPORTED: return "valid request not supported by this build";
        case UOE_ERR_WORKSPACE: return "workspace missing or too small";
        case UOE_ERR_DEVICE: return "kernel launch failed";
        case UOE_ERR_SCRATCH_LIMIT: return "request needs more than the fixed scratch of the entry point that allocates nothing";
        default: return "unknown status";
    }
}

size_t uoe_workspace_bytes(const uoe_block_desc *smha, const uoe_block_desc *uome)
{
    size_t total = 0;
    if (smha) {
        if (check_desc(smha, DESC_SMHA) != UOE_OK) return 0;
        total += route_ws(smha->b, smha->l, smha->d, smha->n, smha->m, smha->dtype == UOE_BF16).total + smha_ws(smha).total +
                 routing_buf(smha, smha->m, smha->c).total;
    }
    if (uome) {
        if (check_desc(uome, DESC_UOME) != UOE_OK) return 0;
        total += route_ws(uome->b, uome->l, uome->d, uome->n, uome->m, uome->dtype == UOE_BF16).total + uome_ws(uome) +
                 routing_buf(uome, uome->m, uome->c).total;
    }
    if (smha && uome) total += up((size_t)smha->b * smha->l * smha->d * elem_size(smha->dtype));  // u
    return total;
}

int uoe_route(const uoe_block_desc *blk, const void *x, const void *w_expert, const void *w_b,
              const void *w_a, const float *noise_expert, const float *noise_patch,
              int32_t *expert_idx, float *expert_gate, int32_t *patch_idx, float *patch_gate,
              void *ws, size_t ws_bytes, void *hip_stream)
{
    const int rc = check_desc(blk, DESC_ROUTE);
    if (rc != UOE_OK) return rc;
    return do_route(blk, blk->m, blk->c, x, w_expert, w_b, w_a, noise_expert, noise_patch, expert_idx,
                    expert_gate, patch_idx, patch_gate, ws, ws_bytes, static_cast<hipStream_t>(hip_stream));
}

int uoe_route_static(const uoe_block_desc *blk, const void *x, const void *w_expert, const void *w_b,
                     const void *w_a, const float *noise_expert, const float *noise_patch,
                     int32_t *expert_idx, float *expert_gate, int32_t *patch_idx, float *patch_gate,
                     void *hip_stream)
{
    const int rc = check_desc(blk, DESC_ROUTE);
    if (rc != UOE_OK) return rc;
    const RouteWs w = route_ws(blk->b, blk->l, blk->d, blk->n, blk->m, blk->dtype == UOE_BF16);
    if (w.total > (size_t)UOE_ROUTE_STATIC_SCRATCH_BYTES) return UOE_ERR_SCRATCH_LIMIT;
    void *ws = nullptr;
    const int sc = static_scratch(&ws);
    if (sc != UOE_OK) return sc;
    // every partial the kernels read from the scratch was written by this same call: nothing to clear
    return do_route(blk, blk->m, blk->c, x, w_expert, w_b, w_a, noise_expert, noise_patch, expert_idx,
                    expert_gate, patch_idx, patch_gate, ws, UOE_ROUTE_STATIC_SCRATCH_BYTES, static_cast<hipStream_t>(hip_stream));
}

int uoe_gather(const uoe_block_desc *blk, const void *x, const int32_t *expert_idx,
               const int32_t *patch_idx, void *h, void *hip_stream)
{
    const int rc = check_desc(blk, DESC_ROUTE);
    if (rc != UOE_OK) return rc;
    if (!x || !expert_idx || !patch_idx || !h || !aligned16(x) || !aligned16(h) || h == x)
        return UOE_ERR_INVALID_ARG;
    GatherArgs a{};
    a.x = x; a.expert_idx = expert_idx; a.patch_idx = patch_idx; a.h = h;
    a.b = blk->b; a.l = blk->l; a.d = blk->d; a.n = blk->n; a.k = blk->k; a.m = blk->m; a.c = blk->c;
    return launch_gather(a, blk->dtype == UOE_BF16, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? UOE_OK : UOE_ERR_DEVICE;
}

int uoe_route_capacity(const uoe_block_desc *blk, const void *x, const void *w_b, const void *w_a,
                       const float *noise_patch, int32_t patch_k, int32_t *capacity, float *load_f,
                       float *load_p, void *ws, size_t ws_bytes, void *hip_stream)
{
    const int rc = check_desc(blk, DESC_ROUTE);
    if (rc != UOE_OK) return rc;
    if (!x || !w_b || !w_a || !capacity || !aligned16(x) || !aligned16(w_b) || !aligned16(w_a))
        return UOE_ERR_INVALID_ARG;
    if (patch_k < 1 || patch_k > blk->n) return UOE_ERR_INVALID_ARG;
    if ((size_t)blk->n * blk->d * elem_size(blk->dtype) > 48 * 1024) return UOE_ERR_UNSUPPORTED;
    if ((size_t)blk->n * blk->m * sizeof(float) > 32 * 1024) return UOE_ERR_UNSUPPORTED;  // logits staged in LDS
    const RouteWs w = route_ws(blk->b, blk->l, blk->d, blk->n, blk->m, blk->dtype == UOE_BF16);
    if (!ws || ws_bytes < w.total || !aligned16(ws)) return UOE_ERR_WORKSPACE;

    RouteArgs a{};
    a.x = x; a.w_b = w_b; a.w_a = w_a;
    a.noise_p = noise_patch;
    a.b = blk->b; a.l = blk->l; a.d = blk->d; a.n = blk->n; a.k = blk->n; a.m = blk->m; a.c = blk->m;
    a.tc = w.tc; a.nchunks = w.nchunks; a.tc_d = w.tc_d; a.nchunks_d = w.nchunks_d;
    a.zpart = reinterpret_cast<float *>(at(ws, w.zpart));
    a.gpart = reinterpret_cast<float *>(at(ws, w.gpart));
    a.gred = reinterpret_cast<float *>(at(ws, w.gred));
    a.patch_k = patch_k;
    a.capacity = capacity; a.load_f = load_f; a.load_p = load_p;
    return launch_route(a, blk->dtype == UOE_BF16, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? UOE_OK
                                                                                                         : UOE_ERR_DEVICE;
}

int uoe_balance_loss(const uoe_block_desc *blk, const float *load_f, const float *load_p, float alpha, float *loss,
                     float *d_patch_gate, void *hip_stream)
{
    const int rc = check_desc(blk, DESC_ROUTE);
    if (rc != UOE_OK) return rc;
    if (!load_f || (loss && !load_p) || (!loss && !d_patch_gate)) return UOE_ERR_INVALID_ARG;
    if (!(alpha == alpha)) return UOE_ERR_INVALID_ARG;  // NaN
    return launch_balance_loss(load_f, load_p, alpha, loss, d_patch_gate, blk->b, blk->n, blk->m,
                               static_cast<hipStream_t>(hip_stream)) == hipSuccess ? UOE_OK : UOE_ERR_DEVICE;
}

int uoe_smha_forward(const uoe_block_desc *blk, const void *x, const void *wq, const void *wk,
                     const void *wv, const void *wo, const int32_t *expert_idx,
                     const float *expert_gate, const int32_t *patch_idx, const float *patch_gate,
                     void *out, void *ws, size_t ws_bytes, void *hip_stream)
{
    const int rc = check_desc(blk, DESC_SMHA);
    if (rc != UOE_OK) return rc;
    return do_smha(blk, x, wq, wk, wv, wo, expert_idx, expert_gate, patch_idx, patch_gate, nullptr, out, ws, ws_bytes,
                   static_cast<hipStream_t>(hip_stream));
}

int uoe_smha_forward_masked(const uoe_block_desc *blk, const void *x, const void *wq, const void *wk,
                            const void *wv, const void *wo, const int32_t *expert_idx,
                            const float *expert_gate, const int32_t *patch_idx, const float *patch_gate,
                            const uint8_t *pad_mask, void *out, void *ws, size_t ws_bytes, void *hip_stream)
{
    const int rc = check_desc(blk, DESC_SMHA);
    if (rc != UOE_OK) return rc;
    return do_smha(blk, x, wq, wk, wv, wo, expert_idx, expert_gate, patch_idx, patch_gate, pad_mask, out, ws,
                   ws_bytes, static_cast<hipStream_t>(hip_stream));
}

int uoe_smha_forward_steps(const uoe_block_desc *blk, const void *x, const void *wq, const void *wk,
                           const void *wv, const void *wo, const int32_t *expert_idx,
                           const float *expert_gate, const int32_t *patch_idx, const float *patch_gate,
                           const uint8_t *pad_mask, void *out, void *ws, size_t ws_bytes, uint32_t steps,
                           void *hip_stream)
{
    const int rc = check_desc(blk, DESC_SMHA);
    if (rc != UOE_OK) return rc;
    const uint32_t all = UOE_SMHA_STEP_QKV | UOE_SMHA_STEP_ATTENTION | UOE_SMHA_STEP_OUT;
    if (steps == 0 || (steps & ~all)) return UOE_ERR_INVALID_ARG;
    return do_smha(blk, x, wq, wk, wv, wo, expert_idx, expert_gate, patch_idx, patch_gate, pad_mask, out, ws,
                   ws_bytes, static_cast<hipStream_t>(hip_stream), all & ~steps);
}

int uoe_uome_forward(const uoe_block_desc *blk, const void *u, const void *a_in, const void *a_out,
                     const int32_t *expert_idx, const float *expert_gate, const int32_t *patch_idx,
                     const float *patch_gate, void *out, void *ws, size_t ws_bytes, void *hip_stream)
{
    const int rc = check_desc(blk, DESC_UOME);
    if (rc != UOE_OK) return rc;
    return do_uome(blk, u, a_in, a_out, expert_idx, expert_gate, patch_idx, patch_gate, out, ws, ws_bytes,
                   static_cast<hipStream_t>(hip_stream));
}

size_t uoe_uome_backward_workspace_bytes(const uoe_block_desc *blk)
{
    return check_uome_bwd(blk) == UOE_OK ? uome_bwd_ws(blk).total : 0;
}

int uoe_uome_backward(const uoe_block_desc *blk, const void *u, const void *a_in, const void *a_out,
                      const int32_t *expert_idx, const float *expert_gate, const int32_t *patch_idx,
                      const float *patch_gate, const void *d_out, void *d_u, void *d_a_in, void *d_a_out, float *d_gate,
                      float *d_patch_gate, void *ws, size_t ws_bytes, void *hip_stream)
{
    const int rc = check_uome_bwd(blk);
    if (rc != UOE_OK) return rc;
    if (!u || !a_in || !a_out || !expert_idx || !d_out || !d_u || !d_a_in || !d_a_out) return UOE_ERR_INVALID_ARG;
    if ((blk->flags & UOE_FLAG_GATE_EXPERT) && !expert_gate) return UOE_ERR_INVALID_ARG;
    // mode as in uoe_uome_forward: patch_idx given = data selection, else c == m and no patch gate
    if ((patch_idx == nullptr) != (blk->c == blk->m)) return UOE_ERR_INVALID_ARG;
    if (!patch_idx && (blk->flags & UOE_FLAG_GATE_PATCH)) return UOE_ERR_INVALID_ARG;
    if ((blk->flags & UOE_FLAG_GATE_PATCH) && !patch_gate) return UOE_ERR_INVALID_ARG;
    if (!aligned16(u) || !aligned16(a_in) || !aligned16(a_out) || !aligned16(d_out) || !aligned16(d_u) ||
        !aligned16(d_a_in) || !aligned16(d_a_out))
        return UOE_ERR_INVALID_ARG;
    if (d_u == u || d_u == d_out || d_a_in == a_in || d_a_out == a_out) return UOE_ERR_INVALID_ARG;
    const UomeBwdWs w = uome_bwd_ws(blk);
    if (!ws || ws_bytes < w.total || !aligned16(ws)) return UOE_ERR_WORKSPACE;
    UomeBwdArgs a{};
    a.u = u; a.a_in = a_in; a.a_out = a_out; a.d_out = d_out; a.expert_idx = expert_idx; a.expert_gate = expert_gate;
    a.d_u = d_u; a.d_a_in = d_a_in; a.d_a_out = d_a_out; a.d_gate = d_gate;
    a.b = blk->b; a.l = blk->l; a.d = blk->d; a.n = blk->n; a.k = blk->k; a.d_e = blk->width; a.flags = blk->flags;
    if (!uome_bwd_mfma(blk)) {
        a.z = at(ws, w.z); a.dh = at(ws, w.dh);
        a.splits = w.splits;
        a.partial = w.splits > 1 ? reinterpret_cast<float *>(at(ws, w.partial)) : nullptr;
        return launch_uome_backward_generic(a, blk->dtype == UOE_BF16, static_cast<hipStream_t>(hip_stream)) == hipSuccess
                   ? UOE_OK : UOE_ERR_DEVICE;
    }
    a.z = at(ws, w.z); a.dh = at(ws, w.dh); a.dz = at(ws, w.dz);
    a.dz_t = at(ws, w.dz_t); a.h_t = at(ws, w.h_t); a.a_in_t = at(ws, w.a_in_t); a.a_out_t = at(ws, w.a_out_t);
    a.gpart = reinterpret_cast<float *>(at(ws, w.gpart));
    a.partial = reinterpret_cast<float *>(at(ws, w.partial));
    a.gchunks = uome_backward_gate_chunks(blk->l, blk->width);
    a.splits = w.splits;
    a.patch_idx = patch_idx; a.patch_gate = patch_gate; a.d_patch_gate = d_patch_gate;
    a.rt = reinterpret_cast<float *>(at(ws, w.rt)); a.m = blk->m; a.c = blk->c;
    return launch_uome_backward(a, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? UOE_OK : UOE_ERR_DEVICE;
}

size_t uoe_smha_backward_workspace_bytes(const uoe_block_desc *blk)
{
    return check_smha_bwd(blk) == UOE_OK ? smha_bwd_ws(blk).total : 0;
}

int uoe_smha_backward(const uoe_block_desc *blk, const void *x, const uoe_smha_weights *w, const int32_t *expert_idx,
                      const float *expert_gate, const int32_t *patch_idx, const float *patch_gate, const uint8_t *pad_mask,
                      const void *d_out, void *d_x, const uoe_smha_weight_grads *dw, float *d_expert_gate,
                      float *d_patch_gate, void *ws, size_t ws_bytes, void *hip_stream)
{
    const int rc = check_smha_bwd(blk);
    if (rc != UOE_OK) return rc;
    if (!x || !w || !dw || !expert_idx || !patch_idx || !d_out || !d_x) return UOE_ERR_INVALID_ARG;
    if (!w->wq || !w->wk || !w->wv || !w->wo || !dw->d_wq || !dw->d_wk || !dw->d_wv || !dw->d_wo) return UOE_ERR_INVALID_ARG;
    if ((blk->flags & UOE_FLAG_GATE_EXPERT) && !expert_gate) return UOE_ERR_INVALID_ARG;
    if ((blk->flags & UOE_FLAG_GATE_PATCH) && !patch_gate) return UOE_ERR_INVALID_ARG;
    const void *ptrs[] = {x, w->wq, w->wk, w->wv, w->wo, d_out, d_x, dw->d_wq, dw->d_wk, dw->d_wv, dw->d_wo};
    for (const void *p : ptrs)
        if (!aligned16(p)) return UOE_ERR_INVALID_ARG;
    if (d_x == x || d_x == d_out) return UOE_ERR_INVALID_ARG;
    const SmhaBwdWs s = smha_bwd_ws(blk);
    if (!ws || ws_bytes < s.total || !aligned16(ws)) return UOE_ERR_WORKSPACE;

    SmhaBwdArgs a{};
    SmhaArgs &f = a.f;
    f.x = x; f.wq = w->wq; f.wk = w->wk; f.wv = w->wv; f.wo = w->wo;
    f.expert_idx = expert_idx; f.patch_idx = patch_idx;
    f.b = blk->b; f.l = blk->l; f.d = blk->d; f.n = blk->n; f.k = blk->k; f.m = blk->m; f.c = blk->c;
    f.d_h = blk->width; f.flags = blk->flags & UOE_FLAG_CAUSAL;  // the recomputed o carries no gate
    f.rope_dim = blk->rope_dim; f.pad_mask = pad_mask;
    f.keep_v_bf16 = 1;   // the attention gradient kernels take v in bf16
    if (!smha_bwd_mfma(blk)) {
        f.q = at(ws, s.g_q); f.kk = at(ws, s.g_k); f.v = at(ws, s.g_v); f.o = at(ws, s.g_o);
        a.d_out = d_out; a.expert_gate = expert_gate; a.patch_gate = patch_gate; a.flags = blk->flags;
        a.d_x = d_x; a.d_wq = dw->d_wq; a.d_wk = dw->d_wk; a.d_wv = dw->d_wv; a.d_wo = dw->d_wo;
        a.d_expert_gate = d_expert_gate; a.d_patch_gate = d_patch_gate;
        a.do_raw = reinterpret_cast<float *>(at(ws, s.do_raw)); a.dqkv = at(ws, s.dqkv);
        a.rt = reinterpret_cast<float *>(at(ws, s.rt));
        a.probs = reinterpret_cast<float *>(at(ws, s.g_probs)); a.dscores = reinterpret_cast<float *>(at(ws, s.g_dscores));
        a.wt = reinterpret_cast<float *>(at(ws, s.g_wt));
        a.splits = s.g_splits;
        a.partial = s.g_splits > 1 ? reinterpret_cast<float *>(at(ws, s.partial)) : nullptr;
        return launch_smha_backward_generic(a, blk->dtype == UOE_BF16, static_cast<hipStream_t>(hip_stream)) == hipSuccess
                   ? UOE_OK : UOE_ERR_DEVICE;
    }
    f.q = at(ws, s.fwd.q); f.kk = at(ws, s.fwd.k); f.v = at(ws, s.fwd.v); f.o = at(ws, s.fwd.o); f.o_lo = at(ws, s.fwd.o_lo);
    f.lse = reinterpret_cast<float *>(at(ws, s.lse));
    a.d_out = d_out; a.expert_gate = expert_gate; a.patch_gate = patch_gate; a.flags = blk->flags;
    a.d_x = d_x; a.d_wq = dw->d_wq; a.d_wk = dw->d_wk; a.d_wv = dw->d_wv; a.d_wo = dw->d_wo;
    a.d_expert_gate = d_expert_gate; a.d_patch_gate = d_patch_gate;
    a.wo_t = at(ws, s.wo_t); a.wqkv_t = at(ws, s.wqkv_t); a.do_raw = reinterpret_cast<float *>(at(ws, s.do_raw)); a.d_o = at(ws, s.d_o);
    a.o_t = at(ws, s.o_t); a.dqkv = at(ws, s.dqkv); a.dqkv_t = at(ws, s.dqkv_t);
    a.rt = reinterpret_cast<float *>(at(ws, s.rt)); a.dd = reinterpret_cast<float *>(at(ws, s.dd));
    a.partial = reinterpret_cast<float *>(at(ws, s.partial));
    a.splits = smha_backward_splits(blk->b, blk->n, blk->k, blk->c);
    return launch_smha_backward(a, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? UOE_OK : UOE_ERR_DEVICE;
}

size_t uoe_route_backward_workspace_bytes(const uoe_block_desc *blk)
{
    return check_route_bwd(blk) == UOE_OK ? route_bwd_ws(blk).total : 0;
}

int uoe_route_backward(const uoe_block_desc *blk, const void *x, const void *w_expert, const void *w_b, const void *w_a,
                       const float *expert_gate, const float *patch_gate, const float *d_expert_gate,
                       const float *d_patch_gate, void *d_x, void *d_w_expert, void *d_w_b, void *d_w_a, void *ws,
                       size_t ws_bytes, void *hip_stream)
{
    const int rc = check_route_bwd(blk);
    if (rc != UOE_OK) return rc;
    if (!x || !d_x || d_x == x || (!w_expert && !w_b)) return UOE_ERR_INVALID_ARG;
    if ((w_b == nullptr) != (w_a == nullptr)) return UOE_ERR_INVALID_ARG;
    if (w_expert && (!expert_gate || !d_expert_gate || !d_w_expert)) return UOE_ERR_INVALID_ARG;
    if (w_b && (!patch_gate || !d_patch_gate || !d_w_b || !d_w_a)) return UOE_ERR_INVALID_ARG;
    const void *ptrs[] = {x, d_x, w_expert, w_b, w_a, d_w_expert, d_w_b, d_w_a};
    for (const void *p : ptrs)
        if (!aligned16(p)) return UOE_ERR_INVALID_ARG;
    const RouteBwdWs w = route_bwd_ws(blk);
    if (!ws || ws_bytes < w.total || !aligned16(ws)) return UOE_ERR_WORKSPACE;
    RouteBwdArgs a{};
    a.x = x; a.w_e = w_expert; a.w_b = w_b; a.w_a = w_a;
    a.g_e = expert_gate; a.g_p = patch_gate; a.d_g_e = d_expert_gate; a.d_g_p = d_patch_gate;
    a.d_x = d_x; a.d_w_e = d_w_expert; a.d_w_b = d_w_b; a.d_w_a = d_w_a;
    a.b = blk->b; a.l = blk->l; a.d = blk->d; a.n = blk->n; a.m = blk->m;
    a.dz = reinterpret_cast<float *>(at(ws, w.dz)); a.dl = reinterpret_cast<float *>(at(ws, w.dl));
    a.t1 = reinterpret_cast<float *>(at(ws, w.t1)); a.u = reinterpret_cast<float *>(at(ws, w.u));
    a.wb_part = reinterpret_cast<float *>(at(ws, w.wb_part));
    a.wb_tokens = w.wb_tokens; a.wb_chunks = w.wb_chunks;
    return launch_route_backward(a, blk->dtype == UOE_BF16, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? UOE_OK : UOE_ERR_DEVICE;
}

int uoe_uome_up(const uoe_block_desc *blk, const void *u, const void *a_in, const int32_t *expert_idx,
                const float *expert_gate, void *hidden, void *hip_stream)
{
    const int rc = check_desc(blk, DESC_UOME);
    if (rc != UOE_OK) return rc;
    if (blk->c != blk->m || (blk->flags & UOE_FLAG_GATE_PATCH)) return UOE_ERR_UNSUPPORTED;
    if (!u || !a_in || !expert_idx || !hidden || hidden == u) return UOE_ERR_INVALID_ARG;
    if (!aligned16(u) || !aligned16(a_in) || !aligned16(hidden)) return UOE_ERR_INVALID_ARG;
    if ((blk->flags & UOE_FLAG_GATE_EXPERT) && !expert_gate) return UOE_ERR_INVALID_ARG;
    UomeArgs a{};
    a.u = u; a.a_in = a_in; a.expert_idx = expert_idx; a.expert_gate = expert_gate; a.hidden = hidden;
    a.b = blk->b; a.l = blk->l; a.d = blk->d; a.n = blk->n; a.k = blk->k; a.d_e = blk->width;
    a.flags = blk->flags;
    return launch_uome_up(a, blk->dtype == UOE_BF16, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? UOE_OK : UOE_ERR_DEVICE;
}

int uoe_uome_down(const uoe_block_desc *blk, const void *hidden, const void *a_out, const void *u,
                  const int32_t *expert_idx, void *out, void *hip_stream)
{
    const int rc = check_desc(blk, DESC_UOME);
    if (rc != UOE_OK) return rc;
    if (blk->c != blk->m) return UOE_ERR_UNSUPPORTED;
    if (!hidden || !a_out || !expert_idx || !out || out == hidden || out == u) return UOE_ERR_INVALID_ARG;
    if ((blk->flags & UOE_FLAG_RESIDUAL) && !u) return UOE_ERR_INVALID_ARG;
    if (!aligned16(hidden) || !aligned16(a_out) || !aligned16(u) || !aligned16(out)) return UOE_ERR_INVALID_ARG;
    UomeArgs a{};
    a.u = u; a.a_out = a_out; a.expert_idx = expert_idx; a.hidden = const_cast<void *>(hidden); a.out = out;
    a.b = blk->b; a.l = blk->l; a.d = blk->d; a.n = blk->n; a.k = blk->k; a.d_e = blk->width;
    a.flags = blk->flags;
    return launch_uome_down(a, blk->dtype == UOE_BF16, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? UOE_OK : UOE_ERR_DEVICE;
}

int uoe_layer_forward(const uoe_block_desc *smha, const uoe_smha_weights *wa,
                      const float *noise_a_expert, const float *noise_a_patch,
                      const uoe_block_desc *uome, const uoe_uome_weights *wm,
                      const float *noise_m_expert, const void *x, void *out,
                      const uoe_routing_out *routing_a, const uoe_routing_out *routing_m, void *ws,
                      size_t ws_bytes, void *hip_stream)
{
    return uoe_layer_forward_masked(smha, wa, noise_a_expert, noise_a_patch, uome, wm, noise_m_expert, x, nullptr, out,
                                    routing_a, routing_m, ws, ws_bytes, hip_stream);
}

int uoe_layer_forward_masked(const uoe_block_desc *smha, const uoe_smha_weights *wa,
                             const float *noise_a_expert, const float *noise_a_patch,
                             const uoe_block_desc *uome, const uoe_uome_weights *wm,
                             const float *noise_m_expert, const void *x, const uint8_t *pad_mask, void *out,
                             const uoe_routing_out *routing_a, const uoe_routing_out *routing_m, void *ws,
                             size_t ws_bytes, void *hip_stream)
{
    int rc = check_desc(smha, DESC_SMHA);
    if (rc != UOE_OK) return rc;
    rc = check_desc(uome, DESC_UOME);
    if (rc != UOE_OK) return rc;
    if (!wa || !wm || !x || !out || out == x) return UOE_ERR_INVALID_ARG;
    if (smha->b != uome->b || smha->l != uome->l || smha->d != uome->d || smha->dtype != uome->dtype)
        return UOE_ERR_INVALID_ARG;
    const bool uome_ds = uome->c != uome->m;
    if (uome_ds && (!wm->w_b || !wm->w_a)) return UOE_ERR_INVALID_ARG;
    // everything the per-block launches would reject is rejected here, before the first launch
    if (!wa->wq || !wa->wk || !wa->wv || !wa->wo || !wm->a_in || !wm->a_out) return UOE_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(out) || !aligned16(wa->w_expert) || !aligned16(wa->w_b) || !aligned16(wa->w_a) ||
        !aligned16(wa->wq) || !aligned16(wa->wk) || !aligned16(wa->wv) || !aligned16(wa->wo) ||
        !aligned16(wm->w_expert) || !aligned16(wm->w_b) || !aligned16(wm->w_a) || !aligned16(wm->a_in) ||
        !aligned16(wm->a_out))
        return UOE_ERR_INVALID_ARG;
    if ((wa->w_b == nullptr) != (wa->w_a == nullptr) || (wm->w_b == nullptr) != (wm->w_a == nullptr))
        return UOE_ERR_INVALID_ARG;
    if ((!wa->w_expert && smha->k != smha->n) || (!wa->w_b && smha->c != smha->m) ||
        (!wm->w_expert && uome->k != uome->n))
        return UOE_ERR_INVALID_ARG;
    if ((!wa->w_expert && noise_a_expert) || (!wa->w_b && noise_a_patch) || (!wm->w_expert && noise_m_expert))
        return UOE_ERR_INVALID_ARG;
    if (wa->w_b && (size_t)smha->n * smha->d * elem_size(smha->dtype) > 48 * 1024) return UOE_ERR_UNSUPPORTED;
    if (uome_ds && (size_t)uome->n * uome->d * elem_size(uome->dtype) > 48 * 1024) return UOE_ERR_UNSUPPORTED;
    if (!uome_ds && (uome->flags & UOE_FLAG_GATE_PATCH)) return UOE_ERR_INVALID_ARG;
    const size_t need = uoe_workspace_bytes(smha, uome);
    if (!ws || ws_bytes < need || !aligned16(ws)) return UOE_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);

    // workspace: [u][routing A][routing M][route scratch A][smha scratch][route scratch M][uome scratch]
    size_t off = 0;
    void *u = at(ws, off);
    off += up((size_t)smha->b * smha->l * smha->d * elem_size(smha->dtype));
    const RoutingBuf ra = routing_buf(smha, smha->m, smha->c);
    char *rabuf = at(ws, off); off += ra.total;
    const RoutingBuf rm = routing_buf(uome, uome->m, uome->c);
    char *rmbuf = at(ws, off); off += rm.total;
    const size_t route_a_bytes = route_ws(smha->b, smha->l, smha->d, smha->n, smha->m, smha->dtype == UOE_BF16).total;
    void *route_a_ws = at(ws, off); off += route_a_bytes;
    const size_t smha_bytes = smha_ws(smha).total;
    void *smha_scratch = at(ws, off); off += smha_bytes;
    const size_t route_m_bytes = route_ws(uome->b, uome->l, uome->d, uome->n, uome->m, uome->dtype == UOE_BF16).total;
    void *route_m_ws = at(ws, off); off += route_m_bytes;
    void *uome_scratch = at(ws, off);
    const size_t uome_bytes = uome_ws(uome);

    auto pick = [](void *user, char *base, size_t o) -> void * { return user ? user : base + o; };
    int32_t *a_eidx = static_cast<int32_t *>(pick(routing_a ? routing_a->expert_idx : nullptr, rabuf, ra.expert_idx));
    float *a_egate = static_cast<float *>(pick(routing_a ? routing_a->expert_gate : nullptr, rabuf, ra.expert_gate));
    int32_t *a_pidx = static_cast<int32_t *>(pick(routing_a ? routing_a->patch_idx : nullptr, rabuf, ra.patch_idx));
    float *a_pgate = static_cast<float *>(pick(routing_a ? routing_a->patch_gate : nullptr, rabuf, ra.patch_gate));
    int32_t *m_eidx = static_cast<int32_t *>(pick(routing_m ? routing_m->expert_idx : nullptr, rmbuf, rm.expert_idx));
    float *m_egate = static_cast<float *>(pick(routing_m ? routing_m->expert_gate : nullptr, rmbuf, rm.expert_gate));
    int32_t *m_pidx = static_cast<int32_t *>(pick(routing_m ? routing_m->patch_idx : nullptr, rmbuf, rm.patch_idx));
    float *m_pgate = static_cast<float *>(pick(routing_m ? routing_m->patch_gate : nullptr, rmbuf, rm.patch_gate));

    rc = do_route(smha, smha->m, smha->c, x, wa->w_expert, wa->w_b, wa->w_a, noise_a_expert, noise_a_patch,
                  a_eidx, a_egate, a_pidx, a_pgate, route_a_ws, route_a_bytes, st);
    if (rc != UOE_OK) return rc;
    rc = do_smha(smha, x, wa->wq, wa->wk, wa->wv, wa->wo, a_eidx, a_egate, a_pidx, a_pgate, pad_mask, u, smha_scratch,
                 smha_bytes, st);
    if (rc != UOE_OK) return rc;
    // the UoME routers read u, the finished SMHA output
    if (uome_ds) {
        rc = do_route(uome, uome->m, uome->c, u, wm->w_expert, wm->w_b, wm->w_a, noise_m_expert, nullptr, m_eidx,
                      m_egate, m_pidx, m_pgate, route_m_ws, route_m_bytes, st);
        if (rc != UOE_OK) return rc;
        return do_uome(uome, u, wm->a_in, wm->a_out, m_eidx, m_egate, m_pidx, m_pgate, out, uome_scratch, uome_bytes, st);
    }
    // expert-selection mode: one patch = the sample
    rc = do_route(uome, 1, 1, u, wm->w_expert, nullptr, nullptr, noise_m_expert, nullptr, m_eidx, m_egate,
                  nullptr, nullptr, route_m_ws, route_m_bytes, st);
    if (rc != UOE_OK) return rc;
    return do_uome(uome, u, wm->a_in, wm->a_out, m_eidx, m_egate, nullptr, nullptr, out, uome_scratch, uome_bytes, st);
}

// workspace of the layer backward: [u][d_u][gate gradients][the largest of the stages' own scratch]
struct LayerBwdWs {
    size_t u, d_u, d_gate_m, d_pgate_m, d_gate_a, d_pgate_a, stage, stage_bytes, total;
};
// the descriptor the UoME routers ran with: one patch = the sample in expert-selection mode
static uoe_block_desc uome_route_desc(const uoe_block_desc *uome)
{
    uoe_block_desc um = *uome;
    if (um.c == um.m) um.m = um.c = 1;
    return um;
}
static LayerBwdWs layer_bwd_ws(const uoe_block_desc *smha, const uoe_block_desc *uome)
{
    LayerBwdWs w;
    const size_t act = up((size_t)smha->b * smha->l * smha->d * elem_size(smha->dtype));
    const uoe_block_desc um = uome_route_desc(uome);
    size_t off = 0;
    w.u = off; off += act;
    w.d_u = off; off += act;
    w.d_gate_m = off; off += up((size_t)uome->b * uome->n * sizeof(float));
    w.d_pgate_m = off; off += up((size_t)uome->b * uome->n * uome->m * sizeof(float));
    w.d_gate_a = off; off += up((size_t)smha->b * smha->n * sizeof(float));
    w.d_pgate_a = off; off += up((size_t)smha->b * smha->n * smha->m * sizeof(float));
    size_t stage = smha_ws(smha).total;
    const size_t others[] = {uoe_uome_backward_workspace_bytes(uome), uoe_smha_backward_workspace_bytes(smha),
                             uoe_route_backward_workspace_bytes(smha), uoe_route_backward_workspace_bytes(&um)};
    for (size_t v : others) stage = v > stage ? v : stage;
    w.stage = off; w.stage_bytes = stage; off += up(stage);
    w.total = off;
    return w;
}
static int check_layer_bwd(const uoe_block_desc *smha, const uoe_block_desc *uome)
{
    int rc = check_smha_bwd(smha);
    if (rc != UOE_OK) return rc;
    rc = check_uome_bwd(uome);
    if (rc != UOE_OK) return rc;
    if (smha->b != uome->b || smha->l != uome->l || smha->d != uome->d || smha->dtype != uome->dtype) return UOE_ERR_INVALID_ARG;
    const uoe_block_desc um = uome_route_desc(uome);
    if ((rc = check_route_bwd(smha)) != UOE_OK) return rc;
    return check_route_bwd(&um);
}

size_t uoe_layer_backward_workspace_bytes(const uoe_block_desc *smha, const uoe_block_desc *uome)
{
    if (!smha || !uome || check_layer_bwd(smha, uome) != UOE_OK) return 0;
    return layer_bwd_ws(smha, uome).total;
}

int uoe_layer_backward(const uoe_block_desc *smha, const uoe_smha_weights *wa, const uoe_block_desc *uome,
                       const uoe_uome_weights *wm, const void *x, const void *u, const uoe_routing_out *routing_a,
                       const uoe_routing_out *routing_m, const void *d_out, void *d_x, const uoe_smha_weight_grads *dwa,
                       const uoe_router_grads *dra, void *d_a_in, void *d_a_out, const uoe_router_grads *drm, void *ws,
                       size_t ws_bytes, void *hip_stream)
{
    return uoe_layer_backward_masked(smha, wa, uome, wm, x, nullptr, u, routing_a, routing_m, d_out, d_x, dwa, dra, d_a_in,
                                     d_a_out, drm, ws, ws_bytes, hip_stream);
}

int uoe_layer_backward_masked(const uoe_block_desc *smha, const uoe_smha_weights *wa, const uoe_block_desc *uome,
                              const uoe_uome_weights *wm, const void *x, const uint8_t *pad_mask, const void *u,
                              const uoe_routing_out *routing_a, const uoe_routing_out *routing_m, const void *d_out,
                              void *d_x, const uoe_smha_weight_grads *dwa, const uoe_router_grads *dra, void *d_a_in,
                              void *d_a_out, const uoe_router_grads *drm, void *ws, size_t ws_bytes, void *hip_stream)
{
    if (!smha || !uome) return UOE_ERR_INVALID_ARG;
    int rc = check_layer_bwd(smha, uome);
    if (rc != UOE_OK) return rc;
    if (!wa || !wm || !x || !routing_a || !routing_m || !d_out || !d_x || !dwa || !d_a_in || !d_a_out) return UOE_ERR_INVALID_ARG;
    if (!routing_a->expert_idx || !routing_a->patch_idx || !routing_m->expert_idx) return UOE_ERR_INVALID_ARG;
    const bool uome_ds = uome->c < uome->m;
    if (uome_ds && (!wm->w_b || !wm->w_a || !routing_m->patch_idx)) return UOE_ERR_INVALID_ARG;
    if (!uome_ds && (wm->w_b || wm->w_a)) return UOE_ERR_INVALID_ARG;
    const bool route_a = wa->w_expert || wa->w_b, route_m = wm->w_expert || wm->w_b;
    if (route_a && !dra) return UOE_ERR_INVALID_ARG;
    if (route_m && !drm) return UOE_ERR_INVALID_ARG;
    // a router's gate must be an input of its block for its gradient to exist
    if (wa->w_expert && (!(smha->flags & UOE_FLAG_GATE_EXPERT) || !routing_a->expert_gate)) return UOE_ERR_INVALID_ARG;
    if (wa->w_b && (!(smha->flags & UOE_FLAG_GATE_PATCH) || !routing_a->patch_gate)) return UOE_ERR_INVALID_ARG;
    if (wm->w_expert && (!(uome->flags & UOE_FLAG_GATE_EXPERT) || !routing_m->expert_gate)) return UOE_ERR_INVALID_ARG;
    if (wm->w_b && (!(uome->flags & UOE_FLAG_GATE_PATCH) || !routing_m->patch_gate)) return UOE_ERR_INVALID_ARG;
    const LayerBwdWs w = layer_bwd_ws(smha, uome);
    if (!ws || ws_bytes < w.total || !aligned16(ws)) return UOE_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    void *stage = at(ws, w.stage);
    void *d_u = at(ws, w.d_u);
    float *d_gate_m = reinterpret_cast<float *>(at(ws, w.d_gate_m));
    float *d_pgate_m = reinterpret_cast<float *>(at(ws, w.d_pgate_m));
    float *d_gate_a = reinterpret_cast<float *>(at(ws, w.d_gate_a));
    float *d_pgate_a = reinterpret_cast<float *>(at(ws, w.d_pgate_a));

    if (!u) {  // u = SMHA(x) with the given routing
        void *u_ws = at(ws, w.u);
        rc = do_smha(smha, x, wa->wq, wa->wk, wa->wv, wa->wo, routing_a->expert_idx, routing_a->expert_gate,
                     routing_a->patch_idx, routing_a->patch_gate, pad_mask, u_ws, stage, w.stage_bytes, st);
        if (rc != UOE_OK) return rc;
        u = u_ws;
    }
    // UoME block and its router: d_out -> d_u
    rc = uoe_uome_backward(uome, u, wm->a_in, wm->a_out, routing_m->expert_idx, routing_m->expert_gate,
                           uome_ds ? routing_m->patch_idx : nullptr, uome_ds ? routing_m->patch_gate : nullptr, d_out, d_u,
                           d_a_in, d_a_out, d_gate_m, uome_ds ? d_pgate_m : nullptr, stage, w.stage_bytes, hip_stream);
    if (rc != UOE_OK) return rc;
    if (route_m) {
        const uoe_block_desc um = uome_route_desc(uome);
        rc = uoe_route_backward(&um, u, wm->w_expert, wm->w_b, wm->w_a, routing_m->expert_gate, routing_m->patch_gate,
                                d_gate_m, d_pgate_m, d_u, drm->d_w_expert, drm->d_w_b, drm->d_w_a, stage, w.stage_bytes,
                                hip_stream);
        if (rc != UOE_OK) return rc;
    }
    // SMHA block and its routers: d_u -> d_x
    rc = uoe_smha_backward(smha, x, wa, routing_a->expert_idx, routing_a->expert_gate, routing_a->patch_idx,
                           routing_a->patch_gate, pad_mask, d_u, d_x, dwa, d_gate_a, d_pgate_a, stage, w.stage_bytes, hip_stream);
    if (rc != UOE_OK) return rc;
    if (route_a)
        rc = uoe_route_backward(smha, x, wa->w_expert, wa->w_b, wa->w_a, routing_a->expert_gate, routing_a->patch_gate,
                                d_gate_a, d_pgate_a, d_x, dra->d_w_expert, dra->d_w_b, dra->d_w_a, stage, w.stage_bytes,
                                hip_stream);
    return rc;
}

int uoe_probe_copy(const void *src, void *dst, size_t bytes, void *hip_stream)
{
    if (!src || !dst || src == dst || !aligned16(src) || !aligned16(dst) || (bytes & 15)) return UOE_ERR_INVALID_ARG;
    return launch_probe_copy(src, dst, bytes, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? UOE_OK : UOE_ERR_DEVICE;
}

int uoe_probe_read(const void *src, size_t bytes, uint32_t *sink, void *hip_stream)
{
    if (!src || !sink || !aligned16(src) || (bytes & 15)) return UOE_ERR_INVALID_ARG;
    return launch_probe_read(src, bytes, sink, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? UOE_OK : UOE_ERR_DEVICE;
}

int uoe_probe_mfma(const void *operands, int32_t iters, float *sink, double *flops, void *hip_stream)
{
    if (!operands || !sink || !aligned16(operands) || iters < 1) return UOE_ERR_INVALID_ARG;
    // blocks x 4 waves x iters x 8 MFMAs of 32x32x16 (2*32*32*16 FLOP each)
    if (flops) *flops = (double)PROBE_MFMA_BLOCKS * 4.0 * iters * 8.0 * (2.0 * 32 * 32 * 16);
    return launch_probe_mfma(operands, iters, sink, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? UOE_OK : UOE_ERR_DEVICE;
}

}  // extern "C"

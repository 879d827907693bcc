// MFMA grouped GEMM engine for bf16 storage (gfx950): C[M,N] = A[M,K] * B[K,N] per group, fp32
// accumulation in v_mfma_f32_32x32x16_bf16, any problem from problems.h.
//
// Tiling.  A workgroup of WAVES_M x WAVES_N wavefronts owns a BM x BN output tile; each wave owns
// (BM/WAVES_M) x (BN/WAVES_N), a TM x TN grid of 32x32 MFMA tiles.  K advances in steps of BK
// (32 or 64) through double-buffered LDS: the global loads of step t+1 are issued before the
// MFMAs of step t and land in the other buffer, one barrier per step.
//
// Addressing.  K is a concatenation of segments of length kseg() (one expert's slice, or all of
// K).  Row and column base pointers are resolved through the routing indices once per segment
// and kept in registers; inside a segment a tile is base + offset.
//
// Operand layout.  The MFMA wants, per lane, 8 K-consecutive values of one row of its first
// operand and of one column of its second.  Activations A are [M,K] with K contiguous: a 16-byte
// LDS read of a row is already a fragment.  Weights B are [K,N] with N contiguous (the paper's
// [n,d,width] layout); they are copied to LDS as they are, [k][n], and the fragments are taken
// with the gfx950 transposing LDS read (ds_read_b64_tr_b16): in a group of 16 lanes, lane j points
// at row k0 + j/4, columns c0 + 4*(j%4)..+3, and lane i receives column c0 + i, rows k0..k0+3.
// The product is computed transposed, D = B^T A^T (weights as the first MFMA operand), so that an
// accumulator lane is one output ROW and its registers run along N in groups of four: the
// epilogue can then hand 8-byte row pieces to LDS and write 16-byte row pieces to memory.
//
// LDS pitches.  A rows are padded to BK+8 elements (16-byte fragment reads of 16 consecutive rows
// hit 64 distinct banks).  B rows are padded so that the pitch in dwords is 16 or 48 mod 64: the
// four 64-byte row pieces a half-wave touches in one transposing read are then bank-disjoint.
//
// Requirements (checked by the callers): kseg() % BK == 0, N segments multiples of 8.  M and N
// tails are masked.
#pragma once
#include <type_traits>
#include <utility>
#include <type_traits>
#include "common.h"

namespace uoe {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef s16x4_t __attribute__((address_space(3))) * lds_s16x4_ptr;

// 4 K-consecutive values of one column from a [k][n] LDS tile (see the header comment)
__device__ __forceinline__ uint2 lds_read_tr4(const uint16_t *p)
{
    const s16x4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
    return __builtin_bit_cast(uint2, v);
}

typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// two fp32 -> packed bf16, round to nearest even (one v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ uint32_t pack2_bf16(float a, float b)
{
    const f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__host__ __device__ constexpr int largest_divisor_upto(int n, int cap)
{
    int b = cap < n ? cap : n;
    while (n % b) --b;
    return b;
}

// Per-column factors of a tile, one per 8-column group, fetched by the whole workgroup before the
// K loop (the lookups behind col_scale are dependent global loads: taken per column group inside
// the epilogue they would serialise their latency).  The caller's next barrier publishes them.
template <typename P, int BN>
__device__ __forceinline__ void fill_col_scale(const P &p, float *coltab, int g, int n0, int N, int tid, int nthreads)
{
    if constexpr (P::kColScale) {
        for (int c = tid; c < BN / 8; c += nthreads) {
            const int col = n0 + c * 8;
            coltab[c] = p.col_scale(g, col < N ? col : 0);
        }
    }
}

// Epilogue of one wave.  acc is the transposed-product accumulator of a TM x TN grid of 32x32
// tiles: register q of lane (lr, lh) in tile (i, j) is output row i*32 + lr, column
// j*32 + (q/4)*8 + lh*4 + q%4 of the wave tile.  The wave stages its tile in LDS (stage: WM rows
// of SPITCH elements, private to the wave) and then moves 16-byte pieces of rows to memory,
// residual pieces loaded a batch ahead of the stores.  wcol0 = first column of the wave tile
// inside the workgroup tile (indexes coltab); (grow0, gcol0) = its global position.
// Per-row factors of the rows this lane owns in the epilogue (rows i*32 + lane%32 of the wave tile),
// fetched before the K loop like the column factors.
template <typename P, int TM>
__device__ __forceinline__ void load_row_scale(const P &p, float (&rs)[TM], int g, int grow0, int M, int lane)
{
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        rs[i] = 1.0f;
        if constexpr (P::kRowScale) {
            const int row = grow0 + i * 32 + (lane & 31);
            rs[i] = p.row_scale(g, row < M ? row : M - 1);
        }
    }
}

// problems that store fp32 tiles straight from the accumulators declare kF32Out and put4_f32
template <typename P, typename = void> struct writes_f32 {
    static constexpr bool value = false;
};
template <typename P> struct writes_f32<P, std::void_t<decltype(P::kF32Out)>> {
    static constexpr bool value = P::kF32Out;
};

// problems that store some column blocks as fp16 instead of bf16 declare f16_col(column)
template <typename P, typename = void> struct has_f16_cols {
    static constexpr bool value = false;
};
template <typename P> struct has_f16_cols<P, std::void_t<decltype(&P::f16_col)>> {
    static constexpr bool value = true;
};
// two fp32 -> packed fp16, round to nearest even
__device__ __forceinline__ uint32_t pack2_f16_rn(float a, float b)
{
    const _Float16 ha = (_Float16)a, hb = (_Float16)b;
    return (uint32_t)__builtin_bit_cast(uint16_t, ha) | ((uint32_t)__builtin_bit_cast(uint16_t, hb) << 16);
}

template <typename P, typename = void> struct streams_once : std::false_type {};
template <typename P> struct streams_once<P, std::void_t<decltype(std::declval<P>().once)>> : std::true_type {};

// second half of the epilogue: the staged wave tile back out of LDS in 16-byte pieces, the residual
// added, the pieces stored (ONCE: through the problem's non-temporal accessors)
template <typename P, int TM, int TN, int SPITCH, bool ONCE>
__device__ __forceinline__ void wave_write_out(const P &p, uint16_t (*stage)[SPITCH], int g, int grow0, int gcol0, int M, int N, int lane)
{
    constexpr int WM = TM * 32, WN = TN * 32;
    constexpr int WC = WN / 8;           // 16-byte pieces per staged row
    constexpr int NPIECE = (WM * WC) / 64;
    constexpr int BATCH = largest_divisor_upto(NPIECE, 8);
    const bool res = p.has_residual();
#pragma unroll
    for (int t0 = 0; t0 < NPIECE; t0 += BATCH) {
        uint4 r[BATCH];
        if (res) {
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int c = lane + (t0 + u) * 64;
                const int grow = grow0 + c / WC, gcol = gcol0 + (c % WC) * 8;
                if constexpr (streams_once<P>::value)
                    r[u] = (grow < M && gcol < N) ? p.template res8_as<ONCE>(g, grow, gcol) : make_uint4(0, 0, 0, 0);
                else r[u] = (grow < M && gcol < N) ? p.res8(g, grow, gcol) : make_uint4(0, 0, 0, 0);
            }
        }
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int c = lane + (t0 + u) * 64;
            const int row = c / WC, pc = c % WC;
            const int grow = grow0 + row, gcol = gcol0 + pc * 8;
            uint4 piece = *reinterpret_cast<const uint4 *>(&stage[row][pc * 8]);
            if (res) piece = add8_bf16(piece, r[u]);
            if (grow < M && gcol < N) {
                if constexpr (streams_once<P>::value) p.template put8_as<ONCE>(g, grow, gcol, piece);
                else p.put8(g, grow, gcol, piece);
            }
        }
    }
}

template <typename P, int TM, int TN, int SPITCH>
__device__ __forceinline__ void wave_epilogue(const P &p, f32x16_t (&acc)[TM][TN], uint16_t (*stage)[SPITCH], const float *coltab,
                                              const float (&rs)[TM], int g, int grow0, int gcol0, int wcol0, int M, int N,
                                              int lane)
{
    constexpr int WM = TM * 32, WN = TN * 32;
    const int lr = lane & 31, lh = lane >> 5;
    if constexpr (writes_f32<P>::value) {
        // a lane holds 4 consecutive columns of one row per register quad: 16-byte stores; the two
        // half-waves and the four quads of a row complete its 128-byte line in L2
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int grow = grow0 + i * 32 + lr;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int qg = 0; qg < 4; ++qg) {
                    const int gcol = gcol0 + j * 32 + qg * 8 + lh * 4;
                    if (grow < M && gcol < N)
                        p.put4_f32(g, grow, gcol, make_float4(acc[i][j][qg * 4 + 0], acc[i][j][qg * 4 + 1],
                                                              acc[i][j][qg * 4 + 2], acc[i][j][qg * 4 + 3]));
                }
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int qg = 0; qg < 4; ++qg) {
            const int cl = j * 32 + qg * 8 + lh * 4;  // first of 4 consecutive columns, wave-local
            float sc = 1.0f;
            if constexpr (P::kColScale) sc = coltab[(wcol0 + cl) >> 3];
            bool half = false;   // uniform over the wave: a column block's format
            if constexpr (has_f16_cols<P>::value) half = p.f16_col(gcol0 + j * 32 + qg * 8);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const float s2 = P::kRowScale ? sc * rs[i] : sc;
                const float e0 = p.epi(acc[i][j][qg * 4 + 0], s2), e1 = p.epi(acc[i][j][qg * 4 + 1], s2);
                const float e2 = p.epi(acc[i][j][qg * 4 + 2], s2), e3 = p.epi(acc[i][j][qg * 4 + 3], s2);
                const uint32_t w0 = half ? pack2_f16_rn(e0, e1) : pack2_bf16(e0, e1);
                const uint32_t w1 = half ? pack2_f16_rn(e2, e3) : pack2_bf16(e2, e3);
                *reinterpret_cast<uint2 *>(&stage[i * 32 + lr][cl]) = make_uint2(w0, w1);
            }
        }
    // no workgroup barrier: a wave reads back only what it staged itself, and the LDS executes one
    // wave's instructions in order
    __builtin_amdgcn_wave_barrier();
    // Problems with a `once` member choose per launch whether the residual read and the output store carry
    // the non-temporal hint; the choice is made here, once per wave, so that each version keeps its
    // batch of residual loads in flight (a test per access would put a branch between them).
    if constexpr (streams_once<P>::value) {
        if (p.once) wave_write_out<P, TM, TN, SPITCH, true>(p, stage, g, grow0, gcol0, M, N, lane);
        else wave_write_out<P, TM, TN, SPITCH, false>(p, stage, g, grow0, gcol0, M, N, lane);
    } else {
        wave_write_out<P, TM, TN, SPITCH, false>(p, stage, g, grow0, gcol0, M, N, lane);
    }
}

// smallest pad (in dwords) that makes (cols/2 + pad) % 64 equal to 16 or 48
__host__ __device__ constexpr int b_pitch_dwords(int cols)
{
    int p = cols / 2;
    while ((p % 64) != 16 && (p % 64) != 48) p += 4;
    return p;
}

// Workgroup order.  The grid is one-dimensional; hardware deals consecutive workgroup ids
// round-robin over the 8 XCDs (each with its own L2).  Id L therefore maps to tile
// (L % 8) * ceil(tiles / 8) + L / 8, with tiles numbered n-tile fastest, then m-tile, then group:
// every XCD works on one contiguous run of tiles, i.e. a few row-tiles of A times all column
// tiles, so an A row-tile and the group's weight slices are fetched into one L2 only.
struct TileGrid {
    int n_tiles, m_tiles, total, per_xcd;
};

template <typename P, int BM, int BN, int BK, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(WAVES_M *WAVES_N * 64) void gemm_mfma_kernel(P p, TileGrid tg)
{
    constexpr int NT = WAVES_M * WAVES_N * 64;
    constexpr int APITCH = BK + 8;                     // A row pitch in elements
    constexpr int BPITCH = 2 * b_pitch_dwords(BN);     // B row pitch in elements
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int KC = BK / 8;                         // 16-byte chunks per A row
    constexpr int A_CHUNKS = BM * KC;
    constexpr int A_PER_T = (A_CHUNKS + NT - 1) / NT;
    constexpr int NC = BN / 8;                         // 16-byte chunks per B row
    constexpr int B_CHUNKS = BK * NC;
    constexpr int B_PER_T = (B_CHUNKS + NT - 1) / NT;
    constexpr int SPITCH = WN + 8;                     // epilogue staging pitch in elements
    constexpr int A_BYTES = 2 * BM * APITCH * 2, B_BYTES = 2 * BK * BPITCH * 2;
    constexpr int S_BYTES = (NT / 64) * WM * SPITCH * 2;
    constexpr int LDS_BYTES = (A_BYTES + B_BYTES) > S_BYTES ? (A_BYTES + B_BYTES) : S_BYTES;
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be made of 32x32 MFMA tiles");
    static_assert(BK == 32 || BK == 64, "BK is 32 or 64");
    static_assert(BN % 8 == 0, "BN is a multiple of 8");

    __shared__ __align__(16) unsigned char lds_raw[LDS_BYTES];
    uint16_t(*As)[BM][APITCH] = reinterpret_cast<uint16_t(*)[BM][APITCH]>(lds_raw);
    uint16_t(*Bs)[BK][BPITCH] = reinterpret_cast<uint16_t(*)[BK][BPITCH]>(lds_raw + A_BYTES);
    __shared__ float coltab[BN / 8];

    const int tile = (blockIdx.x & 7) * tg.per_xcd + (blockIdx.x >> 3);
    if (tile >= tg.total) return;
    const int g = tile / (tg.n_tiles * tg.m_tiles);
    const int rem = tile - g * (tg.n_tiles * tg.m_tiles);
    const int mt = rem / tg.n_tiles, nt = rem - mt * tg.n_tiles;
    const int M = p.rows(g), N = p.ncols(), K = p.kdim(g), KSEG = p.kseg();
    const int m0 = mt * BM, n0 = nt * BN;
    if (m0 >= M) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
    const int lr = lane & 31, lh = lane >> 5;
    const long bstride = p.b_stride();

    fill_col_scale<P, BN>(p, coltab, g, n0, N, tid, NT);  // published by the barrier before the K loop
    float rs[TM];
    load_row_scale<P, TM>(p, rs, g, m0 + wm0, M, lane);

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

    // per-thread load assignments and their per-segment base pointers
    const uint16_t *a_base[A_PER_T];
    const uint16_t *b_base[B_PER_T];
    auto resolve_segment = [&](int seg) {
#pragma unroll
        for (int i = 0; i < A_PER_T; ++i) {
            const int c = tid + i * NT;
            const int row = c / KC, kc = c % KC;
            a_base[i] = (c < A_CHUNKS && m0 + row < M)
                            ? reinterpret_cast<const uint16_t *>(p.a_seg_ptr(g, m0 + row, seg)) + kc * 8
                            : nullptr;
        }
#pragma unroll
        for (int i = 0; i < B_PER_T; ++i) {
            const int c = tid + i * NT;
            const int row = c / NC, nc = c % NC;
            b_base[i] = (c < B_CHUNKS && n0 + nc * 8 < N)
                            ? reinterpret_cast<const uint16_t *>(p.b_seg_ptr(g, seg, n0 + nc * 8)) + (long)row * bstride
                            : nullptr;
        }
    };

    uint4 a_reg[A_PER_T], b_reg[B_PER_T];
    auto load_global = [&](int off) {  // tile at offset `off` inside the current segment
#pragma unroll
        for (int i = 0; i < A_PER_T; ++i) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (a_base[i]) v = *reinterpret_cast<const uint4 *>(a_base[i] + off);
            a_reg[i] = v;
        }
#pragma unroll
        for (int i = 0; i < B_PER_T; ++i) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (b_base[i]) v = *reinterpret_cast<const uint4 *>(b_base[i] + (long)off * bstride);
            b_reg[i] = v;
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_PER_T; ++i) {
            const int c = tid + i * NT;
            if (c < A_CHUNKS) *reinterpret_cast<uint4 *>(&As[buf][c / KC][(c % KC) * 8]) = a_reg[i];
        }
#pragma unroll
        for (int i = 0; i < B_PER_T; ++i) {
            const int c = tid + i * NT;
            if (c < B_CHUNKS) *reinterpret_cast<uint4 *>(&Bs[buf][c / NC][(c % NC) * 8]) = b_reg[i];
        }
    };

    const int KT = K / BK;
    int nseg_next = 0, noff = 0;  // segment / offset of the next tile to fetch
    auto fetch_next = [&]() {
        if (noff == 0) resolve_segment(nseg_next);
        load_global(noff);
        noff += BK;
        if (noff == KSEG) {
            noff = 0;
            ++nseg_next;
        }
    };
    if (KT > 0) {
        fetch_next();
        store_lds(0);
    }
    __syncthreads();
    // transposing-read lane roles: group gl = lane/16 -> column half (gl & 1), k half (gl >> 1 == lh)
    const int tr_row = lh * 8 + ((lane & 15) >> 2);
    const int tr_col = ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) fetch_next();
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8_t af[TM], wf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[i] = *reinterpret_cast<const bf16x8_t *>(&As[buf][wm0 + i * 32 + lr][ks * 16 + lh * 8]);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const uint16_t *src = &Bs[buf][ks * 16 + tr_row][wn0 + j * 32 + tr_col];
                const uint2 lo = lds_read_tr4(src);
                const uint2 hi = lds_read_tr4(src + 4 * BPITCH);
                wf[j] = __builtin_bit_cast(bf16x8_t, make_uint4(lo.x, lo.y, hi.x, hi.y));
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j], af[i], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) store_lds(buf ^ 1);
        __syncthreads();
    }

    // Epilogue: the operand buffers are free now (the loop ended on a barrier); each wave stages its
    // own tile there.
    uint16_t(*stage)[SPITCH] = reinterpret_cast<uint16_t(*)[SPITCH]>(lds_raw) + (size_t)wave * WM;
    wave_epilogue<P, TM, TN, SPITCH>(p, acc, stage, coltab, rs, g, m0 + wm0, n0 + wn0, wn0, M, N, lane);
}

template <typename P, int BM, int BN, int BK, int WAVES_M, int WAVES_N>
static hipError_t launch_gemm_mfma(const P &p, int groups, int max_rows, int ncols, hipStream_t st)
{
    if (groups <= 0 || max_rows <= 0 || ncols <= 0) return hipSuccess;
    TileGrid tg;
    tg.n_tiles = (ncols + BN - 1) / BN;
    tg.m_tiles = (max_rows + BM - 1) / BM;
    const long total = (long)tg.n_tiles * tg.m_tiles * groups;
    if (total > (1L << 28)) return hipErrorInvalidValue;
    tg.total = (int)total;
    tg.per_xcd = (tg.total + 7) / 8;
    hipLaunchKernelGGL((gemm_mfma_kernel<P, BM, BN, BK, WAVES_M, WAVES_N>), dim3(tg.per_xcd * 8), dim3(WAVES_M * WAVES_N * 64), 0,
                       st, p, tg);
    return hipGetLastError();
}

}  // namespace uoe

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
// Operand layout.  The MFMA wants, per lane, 8 K-consecutive values of one A row and of one B
// column.  A is [M,K] with K contiguous: a 16-byte global load is already an operand fragment.
// B is [K,N] with N contiguous (the paper's [n,d,width] weight layout), so B is transposed on
// the way into LDS: a thread loads two K-rows of 8 columns and interleaves them in registers into
// eight dwords (k, k+1) per column, stored K-contiguous.  LDS rows are padded to BK+8 elements,
// which makes the 16-byte fragment reads of 16 consecutive rows hit 64 distinct banks.
//
// Requirements (checked by the callers): kseg() % BK == 0, N segments multiples of 8.  M and N
// tails are masked.
#pragma once
#include "common.h"

namespace uoe {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

// low/high halves of two dwords -> one dword: (lo16 of a) | (lo16 of b) << 16, and the high pair
__device__ __forceinline__ uint32_t pack_lo(uint32_t a, uint32_t b) { return (a & 0xFFFFu) | (b << 16); }
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xFFFF0000u); }

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
    constexpr int PITCH = BK + 8;                      // LDS row pitch in elements
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int KC = BK / 8;                         // 16-byte chunks per A row
    constexpr int A_CHUNKS = BM * KC;
    constexpr int A_PER_T = (A_CHUNKS + NT - 1) / NT;
    constexpr int KPAIRS = BK / 2;
    constexpr int B_JOBS = KPAIRS * (BN / 8);          // (k pair, 8 columns) jobs in a B tile
    constexpr int B_PER_T = (B_JOBS + NT - 1) / NT;
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be made of 32x32 MFMA tiles");
    static_assert(BK == 32 || BK == 64, "BK is 32 or 64");

    __shared__ __align__(16) uint16_t As[2][BM][PITCH];
    __shared__ __align__(16) uint16_t Bs[2][BN][PITCH];

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
            const int job = tid + i * NT;
            const int kp = job % KPAIRS, nc = job / KPAIRS;
            b_base[i] = (job < B_JOBS && n0 + nc * 8 < N)
                            ? reinterpret_cast<const uint16_t *>(p.b_seg_ptr(g, seg, n0 + nc * 8)) + (long)(2 * kp) * bstride
                            : nullptr;
        }
    };

    uint4 a_reg[A_PER_T];
    uint4 b_reg[B_PER_T][2];
    auto load_global = [&](int off) {  // tile at offset `off` inside the current segment
#pragma unroll
        for (int i = 0; i < A_PER_T; ++i) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (a_base[i]) v = *reinterpret_cast<const uint4 *>(a_base[i] + off);
            a_reg[i] = v;
        }
#pragma unroll
        for (int i = 0; i < B_PER_T; ++i) {
            uint4 r0 = make_uint4(0, 0, 0, 0), r1 = r0;
            if (b_base[i]) {
                const uint16_t *src = b_base[i] + (long)off * bstride;
                r0 = *reinterpret_cast<const uint4 *>(src);
                r1 = *reinterpret_cast<const uint4 *>(src + bstride);
            }
            b_reg[i][0] = r0;
            b_reg[i][1] = r1;
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
            const int job = tid + i * NT;
            if (job < B_JOBS) {
                const int kp = job % KPAIRS, nc = job / KPAIRS;
                const uint4 r0 = b_reg[i][0], r1 = b_reg[i][1];
                uint32_t *d0 = reinterpret_cast<uint32_t *>(&Bs[buf][nc * 8][2 * kp]);
                constexpr int RP = PITCH / 2;  // row pitch in dwords
                d0[0 * RP] = pack_lo(r0.x, r1.x);
                d0[1 * RP] = pack_hi(r0.x, r1.x);
                d0[2 * RP] = pack_lo(r0.y, r1.y);
                d0[3 * RP] = pack_hi(r0.y, r1.y);
                d0[4 * RP] = pack_lo(r0.z, r1.z);
                d0[5 * RP] = pack_hi(r0.z, r1.z);
                d0[6 * RP] = pack_lo(r0.w, r1.w);
                d0[7 * RP] = pack_hi(r0.w, r1.w);
            }
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
    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) fetch_next();
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8_t af[TM], bf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[i] = *reinterpret_cast<const bf16x8_t *>(&As[buf][wm0 + i * 32 + lr][ks * 16 + lh * 8]);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bf[j] = *reinterpret_cast<const bf16x8_t *>(&Bs[buf][wn0 + j * 32 + lr][ks * 16 + lh * 8]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) store_lds(buf ^ 1);
        __syncthreads();
    }

    // epilogue: accumulator register q of lane (lr, lh) is row (q/4)*8 + lh*4 + q%4, column lr
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn0 + j * 32 + lr;
        if (col >= N) continue;
        const auto cc = p.col_ctx(g, col);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int row = m0 + wm0 + i * 32 + (q >> 2) * 8 + lh * 4 + (q & 3);
                if (row < M) p.store(g, row, col, acc[i][j][q], cc);
            }
        }
    }
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

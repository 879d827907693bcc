// Pipelined MFMA grouped GEMM engine for bf16 storage (gfx950), for the large contractions.
// Same contract and the same MFMA/epilogue arrangement as gemm_mfma.h (transposed product,
// weights read from a [k][n] LDS tile with the transposing LDS read, LDS-staged 16-byte stores);
// what differs is how operands reach LDS and how deep the prefetch is:
//
//  * Operand tiles go from global memory straight into LDS (global_load_lds_dwordx4: 16 bytes per
//    lane, the 64 lanes of one instruction fill 1 KiB of consecutive LDS bytes starting at M0).
//    No registers are held by loads in flight and no LDS store instructions are issued, so a tile
//    can have STAGES-1 K-steps of loads outstanding while the MFMAs of the current step run.
//  * Since the LDS side of such a load is fixed (lane -> consecutive 16-byte slots) rows cannot be
//    padded.  Bank conflicts are avoided by permuting, per row, WHICH 16-byte chunk of the global
//    row a slot receives (each lane supplies its own global address, so this costs nothing):
//      A tile [BM][BK]:  slot (r, pos) holds chunk pos ^ ((r / (16/CA)) % CA),  CA = BK/8 chunks/row;
//                        the 16 rows a 16-lane phase of a 16-byte fragment read touches then cover
//                        all 64 banks once.
//      B tile [BK][BN]:  the four 64-byte row pieces (rows k0..k0+3) a half-wave touches in one
//                        transposing read must land in four different 16-bank groups.  With a row
//                        of 256*i bytes (BN % 128 == 0) slot (r, pos) holds chunk
//                        pos ^ ((r & 3) << 2); with a row of 256*i + 128 bytes (BN % 128 == 64)
//                        odd and even rows already differ by 32 banks and slot (r, pos) holds
//                        chunk pos ^ (((r >> 1) & 1) << 2).
//  * The compiler cannot see these loads (they are inline assembly), so their completion is
//    waited for by hand: loads complete in issue order, and at the top of K-step t the wave waits
//    until at most the loads of the STAGES-2 younger steps are outstanding (s_waitcnt vmcnt), then
//    the workgroup barrier makes every wave's part of step t visible and at the same time frees
//    the buffer of step t-1 for the loads of step t+STAGES-1.  One barrier per K-step.
//    No other vector-memory instruction may be issued between the first load and the end of the
//    K loop: a compiler-inserted wait for it would drain the whole pipeline.  Per-segment routing
//    lookups are therefore taken once, before the loop, into a small LDS table (seg_ctx).
//
// Requirements (checked by the callers): kseg() % BK == 0, N % 8 == 0, at most 128 K segments; BN a
// multiple of 64 and both operand tiles a whole number of load instructions per wave.  M and N tails are handled by clamping the load addresses to a valid row / chunk
// of the same tile (the results of clamped rows and columns are never stored).
#pragma once
#include "gemm_mfma.h"
#include <type_traits>

namespace uoe {

#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
// 16 bytes per lane from `gptr` (per lane) to LDS byte address lds_byte + 16*lane (lds_byte
// wave-uniform).  M0 is written and consumed inside the statement.
__device__ __forceinline__ void dma_load16(const void *gptr, uint32_t lds_byte)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_byte), "v"(gptr) : "memory", "m0");
}
#pragma clang diagnostic pop

template <int N> __device__ __forceinline__ void dma_wait()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// OCC = waves per SIMD the register budget is held to (workgroups per CU = OCC * 4 / waves, LDS permitting)
template <typename P, int BM, int BN, int BK, int WAVES_M, int WAVES_N, int STAGES, int OCC>
__global__ __launch_bounds__(WAVES_M *WAVES_N * 64, OCC) void gemm_dma_kernel(P p, TileGrid tg)
{
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int CA = BK / 8, CB = BN / 8;              // 16-byte chunks per A row / B row
    constexpr int ARD = 64 / CA;                         // A rows covered by one load instruction
    constexpr int A_INSTR = BM * CA / 64;                // load instructions that make up the A tile
    // instructions per wave per step; when the A tile has fewer instructions than waves the surplus
    // waves repeat one (same bytes to the same place), so that every wave counts the same loads
    constexpr int A_DMA = (A_INSTR + NW - 1) / NW, B_DMA = BK * CB / (64 * NW);
    constexpr int A_STAGE = BM * BK * 2, B_STAGE = BK * BN * 2, STAGE_BYTES = A_STAGE + B_STAGE;
    constexpr int SPITCH = WN + 8;                       // epilogue staging pitch in elements
    constexpr int S_BYTES = NW * WM * SPITCH * 2;
    constexpr int OPER_BYTES = STAGES * STAGE_BYTES;
    constexpr int LDS_BYTES = OPER_BYTES > S_BYTES ? OPER_BYTES : S_BYTES;
    constexpr int MAX_SEG = 128;
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be made of 32x32 MFMA tiles");
    static_assert(BK == 32 || BK == 64, "BK is 32 or 64");
    static_assert(BN % 64 == 0, "BN is a multiple of 64");
    static_assert((BM * CA) % 64 == 0 && (BK * CB) % (64 * NW) == 0, "tile does not divide into whole load instructions");
    static_assert(A_DMA == 1 || ((NW * ARD) % 16 == 0 && A_INSTR % NW == 0), "the A chunk permutation must not depend on the instruction");
    static_assert(BN / 8 <= NW * 64, "one column-scale entry per thread");
    static_assert(STAGES >= 2 && (STAGES - 2) * (A_DMA + B_DMA) < 64, "vmcnt range");

    __shared__ __align__(1024) unsigned char lds_raw[LDS_BYTES];
    __shared__ uint32_t segtab[MAX_SEG];
    __shared__ float coltab[BN / 8];

    const int tile = (blockIdx.x & 7) * tg.per_xcd + (blockIdx.x >> 3);
    if (tile >= tg.total) return;
    const int g = tile / (tg.n_tiles * tg.m_tiles);
    const int rem = tile - g * (tg.n_tiles * tg.m_tiles);
    const int mt = rem / tg.n_tiles, nt = rem - mt * tg.n_tiles;
    const int M = p.rows(g), N = p.ncols(), KSEG = p.kseg();
    const int m0 = mt * BM, n0 = nt * BN;
    if (m0 >= M) return;
    const int tid = threadIdx.x, lane = tid & 63;
    int K;  // problems whose K segments are found by the workgroup itself fill segtab here
    if constexpr (P::kPrepare) K = p.prepare(g, segtab, tid, NW * 64);
    else K = p.kdim(g);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
    const int lr = lane & 31, lh = lane >> 5;
    const long bstride = p.b_stride();
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds_raw;

    const int nseg = K / KSEG;
    // table entries of this thread (at most one of each), requested now and stored after the first
    // operand loads have been issued
    uint32_t my_seg = 0;
    float my_scale = 1.0f;
    if constexpr (!P::kPrepare) {
        if (tid < nseg && tid < MAX_SEG) my_seg = p.seg_ctx(g, tid);
    }
    if constexpr (P::kColScale) {
        if (tid < BN / 8) my_scale = p.col_scale(g, n0 + tid * 8 < N ? n0 + tid * 8 : 0);
    }
    float rs[TM];
    load_row_scale<P, TM>(p, rs, g, m0 + wm0, M, lane);

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

    // Load roles.  Instruction i of this wave fills block (i*NW + wave) of 1 KiB in the A (or B)
    // part of a stage; lane -> slot (row, pos) inside the block.
    const int a_blk0 = wave % A_INSTR;                              // + i*NW blocks
    const int a_row0 = a_blk0 * ARD + lane / CA, a_pos = lane % CA; // + i*NW*ARD rows
    const int a_chunk = a_pos ^ ((a_row0 / (16 / CA)) % CA);        // independent of i: NW*ARD % 16 == 0
    const uint16_t *a_ptr[A_DMA];
    // When a B row is a whole fraction of one load instruction (and the permutation does not depend
    // on the instruction) a lane keeps one column for all its instructions: one base pointer.
    constexpr bool B_UNIFORM = 64 % CB == 0 && (NW * (64 / CB)) % 4 == 0;
    constexpr int B_PTRS = B_UNIFORM ? 1 : B_DMA;
    constexpr int BRD = B_UNIFORM ? 64 / CB : 0;         // B rows covered by one load instruction
    const uint16_t *b_ptr[B_PTRS];
    auto b_swizzle = [](int row) { return (BN % 128 == 0 ? (row & 3) : ((row >> 1) & 1)) << 2; };
    auto resolve_segment = [&](int seg, uint32_t ctx) {
#pragma unroll
        for (int i = 0; i < A_DMA; ++i) {
            int row = m0 + a_row0 + i * NW * ARD;
            row = row < M ? row : M - 1;
            a_ptr[i] = reinterpret_cast<const uint16_t *>(p.a_ptr_ctx(g, row, seg, ctx)) + a_chunk * 8;
        }
#pragma unroll
        for (int i = 0; i < B_PTRS; ++i) {  // B slots in row-major order: slot -> (row, pos)
            const int slot = (i * NW + wave) * 64 + lane;
            const int row = slot / CB, pos = slot - row * CB;
            int col = n0 + (pos ^ b_swizzle(row)) * 8;
            col = col < N ? col : n0;  // N tail: any valid chunk
            b_ptr[i] = reinterpret_cast<const uint16_t *>(p.b_ptr_ctx(g, seg, col, ctx)) + (long)row * bstride;
        }
    };
    auto issue = [&](int buf, int off) {  // K-step at offset `off` of the current segment -> stage buffer buf
        const uint32_t sbase = lds_base + buf * STAGE_BYTES + wave * 1024;
#pragma unroll
        for (int i = 0; i < A_DMA; ++i) dma_load16(a_ptr[i] + off, sbase + (a_blk0 - wave + i * NW) * 1024);
#pragma unroll
        for (int i = 0; i < B_DMA; ++i)
            dma_load16(b_ptr[B_UNIFORM ? 0 : i] + (long)(off + (B_UNIFORM ? i * NW * BRD : 0)) * bstride,
                       sbase + A_STAGE + i * NW * 1024);
    };

    const int KT = K / BK;
    int nseg_next = 0, noff = 0, nbuf = 0;  // segment / offset / buffer of the next K-step to fetch
    // The first STAGES-1 K-steps are fetched before anything else: their segments' contexts are
    // looked up directly (every lane the same address), so that the first operand bytes are only one
    // dependent load away from the kernel's start.  The lookup tables the loop and the epilogue use
    // are filled afterwards, under those loads, and published by the loop's first barrier.
    auto fetch_next = [&]() {
        if (noff == 0) {
            if constexpr (P::kPrepare) resolve_segment(nseg_next, segtab[nseg_next < MAX_SEG ? nseg_next : 0]);
            else resolve_segment(nseg_next, p.seg_ctx(g, nseg_next));
        }
        issue(nbuf, noff);
        nbuf = nbuf + 1 == STAGES ? 0 : nbuf + 1;
        noff += BK;
        if (noff == KSEG) {
            noff = 0;
            ++nseg_next;
        }
    };
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s)
        if (s < KT) fetch_next();
    if (!P::kPrepare && tid < nseg && tid < MAX_SEG) segtab[tid] = my_seg;
    if (P::kColScale && tid < BN / 8) coltab[tid] = my_scale;

    // fragment read offsets (bytes inside a stage)
    uint32_t a_off[BK / 16], b_off[TN];
    {
        const int swz = (lr / (16 / CA)) % CA;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) a_off[ks] = (wm0 + lr) * (BK * 2) + (((ks * 2 + lh) ^ swz) * 16);
        const int x = (lane & 15) >> 2, colhalf = (lane >> 4) & 1;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int chunk = (wn0 + j * 32) / 8 + colhalf * 2 + ((lane & 3) >> 1);
            b_off[j] = A_STAGE + (lh * 8 + x) * (BN * 2) + ((chunk ^ b_swizzle(x)) * 16) + (lane & 1) * 8;
        }
    }

    // One K-step of matrix work on stage buffer cbuf.  With FETCH, the loads of K-step
    // kt+STAGES-1 are issued in between: one 1 KiB load after every TN MFMAs, so that the
    // address path (64 bytes per clock per CU) drains them in the shadow of the matrix pipe instead
    // of stalling the wave in front of it.
    constexpr int KS = BK / 16;
    constexpr int PIECES = A_DMA + B_DMA, SLOTS = KS * TM, PPS = (PIECES + SLOTS - 1) / SLOTS;
    int cbuf = 0;
    auto k_step = [&](auto fetch) {
        constexpr bool FETCH = decltype(fetch)::value;
        int f_off = 0;
        uint32_t f_base = 0;
        if constexpr (FETCH) {
            if (noff == 0) resolve_segment(nseg_next, segtab[nseg_next < MAX_SEG ? nseg_next : 0]);
            f_off = noff;
            f_base = lds_base + nbuf * STAGE_BYTES + wave * 1024;
            nbuf = nbuf + 1 == STAGES ? 0 : nbuf + 1;
            noff += BK;
            if (noff == KSEG) {
                noff = 0;
                ++nseg_next;
            }
        }
        const unsigned char *st = lds_raw + cbuf * STAGE_BYTES;
        // Fragments are double-buffered in registers: the LDS reads of sub-step ks+1 are issued
        // before the MFMAs of sub-step ks, so their latency is covered by 32*TM*TN cycles of matrix
        // work of this same wave (at one or two waves per SIMD there is little else to cover it).
        // The scheduling fences keep the compiler from sinking the reads back down to their uses.
        bf16x8_t af[2][TM], wf[2][TN];
        auto load_frags = [&](int ks, int slot) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[slot][i] = *reinterpret_cast<const bf16x8_t *>(st + a_off[ks] + i * 32 * BK * 2);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const uint16_t *src = reinterpret_cast<const uint16_t *>(st + b_off[j] + ks * 16 * BN * 2);
                const uint2 lo = lds_read_tr4(src);
                const uint2 hi = lds_read_tr4(src + 4 * BN);
                wf[slot][j] = __builtin_bit_cast(bf16x8_t, make_uint4(lo.x, lo.y, hi.x, hi.y));
            }
        };
        load_frags(0, 0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (ks + 1 < KS) load_frags(ks + 1, (ks + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[ks & 1][j], af[ks & 1][i], acc[i][j], 0, 0, 0);
                if constexpr (FETCH) {
#pragma unroll
                    for (int u = 0; u < PPS; ++u) {
                        const int q = (ks * TM + i) * PPS + u;  // compile-time after unrolling
                        if (q < A_DMA) dma_load16(a_ptr[q < A_DMA ? q : 0] + f_off, f_base + (a_blk0 - wave + q * NW) * 1024);
                        else if (q < PIECES)
                            dma_load16(b_ptr[!B_UNIFORM && q >= A_DMA && q < PIECES ? q - A_DMA : 0] +
                                           (long)(f_off + (B_UNIFORM ? (q - A_DMA) * NW * BRD : 0)) * bstride,
                                       f_base + A_STAGE + (q - A_DMA) * NW * 1024);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        cbuf = cbuf + 1 == STAGES ? 0 : cbuf + 1;
    };
    // K-step kt has landed once at most the loads of the STAGES-2 younger steps are outstanding;
    // the last STAGES-1 steps have nothing left to fetch and simply wait for everything.
    int kt = 0;
    for (; kt + STAGES - 1 < KT; ++kt) {
        dma_wait<(STAGES - 2) * (A_DMA + B_DMA)>();
        __syncthreads();
        k_step(std::true_type{});
    }
    for (; kt < KT; ++kt) {
        dma_wait<0>();
        __syncthreads();
        k_step(std::false_type{});
    }
    __syncthreads();  // every wave has finished reading operands: LDS is free for the epilogue

    uint16_t(*stage)[SPITCH] = reinterpret_cast<uint16_t(*)[SPITCH]>(lds_raw) + (size_t)wave * WM;
    wave_epilogue<P, TM, TN, SPITCH>(p, acc, stage, coltab, rs, g, m0 + wm0, n0 + wn0, wn0, M, N, lane);
}

template <typename P, int BM, int BN, int BK, int WAVES_M, int WAVES_N, int STAGES, int OCC = 1>
static hipError_t launch_gemm_dma(const P &p, int groups, int max_rows, int ncols, hipStream_t st)
{
    if (groups <= 0 || max_rows <= 0 || ncols <= 0) return hipSuccess;
    TileGrid tg;
    tg.n_tiles = (ncols + BN - 1) / BN;
    tg.m_tiles = (max_rows + BM - 1) / BM;
    const long total = (long)tg.n_tiles * tg.m_tiles * groups;
    if (total > (1L << 28)) return hipErrorInvalidValue;
    tg.total = (int)total;
    tg.per_xcd = (tg.total + 7) / 8;
    hipLaunchKernelGGL((gemm_dma_kernel<P, BM, BN, BK, WAVES_M, WAVES_N, STAGES, OCC>), dim3(tg.per_xcd * 8),
                       dim3(WAVES_M * WAVES_N * 64), 0, st, p, tg);
    return hipGetLastError();
}

// Tile choice for contractions without a tuned rule of their own (the backward passes): the large
// tile when it still gives 512 workgroups, short tiles when the launch would not fill the chip.
template <typename P> static hipError_t launch_gemm_dma_auto(const P &p, int groups, int rows, int ncols, int kseg, hipStream_t st)
{
    const long tiles128 = (long)groups * ((rows + 127) / 128) * ((ncols + 127) / 128);
    if (rows > 128 && (long)groups * ((rows + 255) / 256) * ((ncols + 127) / 128) >= 512)
        return launch_gemm_dma<P, 256, 128, 32, 2, 2, 3, 2>(p, groups, rows, ncols, st);
    if (tiles128 < 256 || rows <= 64)
        return kseg % 64 == 0 ? launch_gemm_dma<P, 64, 128, 64, 2, 2, 3, 2>(p, groups, rows, ncols, st)
                              : launch_gemm_dma<P, 64, 128, 32, 2, 2, 4, 2>(p, groups, rows, ncols, st);
    return kseg % 64 == 0 ? launch_gemm_dma<P, 128, 128, 64, 2, 2, 2, 2>(p, groups, rows, ncols, st)
                          : launch_gemm_dma<P, 128, 128, 32, 2, 2, 4, 2>(p, groups, rows, ncols, st);
}

}  // namespace uoe

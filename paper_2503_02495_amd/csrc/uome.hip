// Union-of-MLP-Experts, expert-selection mode (Eq. 38-40 with Eq. 24-26), sample-major:
// a sample's k active experts are column slices of A^I and row slices of A^O, so together they
// are ONE two-layer MLP of hidden width k*d_e for that sample.  GEMM-1 writes the gated
// SiLU hidden activations [l, k*d_e]; GEMM-2 contracts over the stacked K = k*d_e and writes every
// output row once with the residual added: no per-expert partial outputs, no atomics.
#include "common.h"
#include "problems.h"
#include "gemm_generic.h"
#include "gemm_mfma.h"
#include "gemm_dma.h"

namespace uoe {

template <typename T> static hipError_t uome_up_generic(const UomeArgs &a, hipStream_t st)
{
    UomeUpProblem<T> up;
    up.u = static_cast<const T *>(a.u);
    up.a_in = static_cast<const T *>(a.a_in);
    up.expert_idx = a.expert_idx;
    up.expert_gate = (a.flags & F_GATE_EXPERT) ? a.expert_gate : nullptr;
    up.hidden = static_cast<T *>(a.hidden);
    up.l = a.l; up.d = a.d; up.n = a.n; up.kact = a.k; up.d_e = a.d_e;
    return launch_gemm_generic<T>(up, a.b, a.l, a.k * a.d_e, st);
}

template <typename T> static hipError_t uome_down_generic(const UomeArgs &a, hipStream_t st)
{
    UomeDownProblem<T> dn;
    dn.hidden = static_cast<const T *>(a.hidden);
    dn.a_out = static_cast<const T *>(a.a_out);
    dn.u = static_cast<const T *>(a.u);
    dn.expert_idx = a.expert_idx;
    dn.out = static_cast<T *>(a.out);
    dn.l = a.l; dn.d = a.d; dn.n = a.n; dn.kact = a.k; dn.d_e = a.d_e; dn.flags = a.flags;
    return launch_gemm_generic<T>(dn, a.b, a.l, a.d, st);
}

// MFMA path: bf16 storage, and every K segment (d for GEMM-1, d_e for GEMM-2) a multiple of 32
static bool uome_mfma_ok(const UomeArgs &a, bool bf16) { return bf16 && a.d % 32 == 0 && a.d_e % 32 == 0; }

// Tile choice for the pipelined engine.  256x128 tiles (wave tile 128x64, register budget held to two
// workgroups per CU: twice the operand bytes in flight, and a CU is not idle while one of them is
// between tiles) once they fill the chip's 512 workgroup slots; 128x128 tiles with a 64-deep K-step
// otherwise.
static bool uome_big(int b, int l, int ncols)
{
    return l > 128 && (long)b * ((l + 255) / 256) * ((ncols + 127) / 128) >= 512;
}

template <typename P> static hipError_t uome_gemm(const P &p, int b, int l, int ncols, int kseg, hipStream_t st)
{
    if (uome_big(b, l, ncols)) return launch_gemm_dma<P, 256, 128, 32, 2, 2, 3, 2>(p, b, l, ncols, st);
    // 64-row tiles while 128x128 tiles would leave CUs without work
    if (l > 64 && kseg % 64 == 0 && (long)b * ((l + 127) / 128) * ((ncols + 127) / 128) < 256)
        return launch_gemm_dma<P, 64, 128, 64, 2, 2, 3, 2>(p, b, l, ncols, st);
    if (l > 64) return kseg % 64 == 0 ? launch_gemm_dma<P, 128, 128, 64, 2, 2, 2, 2>(p, b, l, ncols, st)
                                      : launch_gemm_dma<P, 128, 128, 32, 2, 2, 4, 2>(p, b, l, ncols, st);
    return launch_gemm_mfma<P, 64, 64, 32, 2, 2>(p, b, l, ncols, st);
}

static hipError_t uome_up_mfma(const UomeArgs &a, hipStream_t st)
{
    UomeUpProblem<bf16_t> up;
    up.u = static_cast<const bf16_t *>(a.u);
    up.a_in = static_cast<const bf16_t *>(a.a_in);
    up.expert_idx = a.expert_idx;
    up.expert_gate = (a.flags & F_GATE_EXPERT) ? a.expert_gate : nullptr;
    up.hidden = static_cast<bf16_t *>(a.hidden);
    up.l = a.l; up.d = a.d; up.n = a.n; up.kact = a.k; up.d_e = a.d_e;
    up.once = stream_once((size_t)a.b * a.l * a.k * a.d_e * sizeof(bf16_t));
    return uome_gemm(up, a.b, a.l, a.k * a.d_e, a.d, st);  // K segment = d
}

static hipError_t uome_down_mfma(const UomeArgs &a, hipStream_t st)
{
    UomeDownProblem<bf16_t> dn;
    dn.hidden = static_cast<const bf16_t *>(a.hidden);
    dn.a_out = static_cast<const bf16_t *>(a.a_out);
    dn.u = static_cast<const bf16_t *>(a.u);
    dn.expert_idx = a.expert_idx;
    dn.out = static_cast<bf16_t *>(a.out);
    dn.l = a.l; dn.d = a.d; dn.n = a.n; dn.kact = a.k; dn.d_e = a.d_e; dn.flags = a.flags;
    dn.once = stream_once((size_t)a.b * a.l * a.d * sizeof(bf16_t));
    return uome_gemm(dn, a.b, a.l, a.d, a.d_e, st);  // K segments = the active experts' d_e rows
}

hipError_t launch_uome_up(const UomeArgs &a, bool bf16, hipStream_t st)
{
    if (uome_mfma_ok(a, bf16)) return uome_up_mfma(a, st);
    return bf16 ? uome_up_generic<bf16_t>(a, st) : uome_up_generic<float>(a, st);
}

hipError_t launch_uome_down(const UomeArgs &a, bool bf16, hipStream_t st)
{
    if (uome_mfma_ok(a, bf16)) return uome_down_mfma(a, st);
    return bf16 ? uome_down_generic<bf16_t>(a, st) : uome_down_generic<float>(a, st);
}

hipError_t launch_uome(const UomeArgs &a, bool bf16, hipStream_t st)
{
    const hipError_t err = launch_uome_up(a, bf16, st);
    return err != hipSuccess ? err : launch_uome_down(a, bf16, st);
}

}  // namespace uoe

// Index selection of Eq. 18 / 24 as a standalone, coalesced copy: every active unit's selected
// patches, in ascending position, into one contiguous [l_a, d] block per unit.
// A patch is a contiguous run of l_p*d elements in x, so the copy moves whole 16-byte vectors;
// one thread per vector, one division per thread to find its patch.  HBM-bound by construction.
#include "common.h"

namespace uoe {

__global__ __launch_bounds__(256) void gather_kernel(GatherArgs a, int vec_per_patch)
{
    const int g = blockIdx.y;  // unit = (sample, slot)
    const int bb = g / a.k, i = clampi(a.expert_idx[g], a.n);
    const long total = (long)a.c * vec_per_patch;
    const int32_t *pid = a.patch_idx + ((size_t)bb * a.n + i) * a.c;
    const uint4 *src = static_cast<const uint4 *>(a.x) + (size_t)bb * a.m * vec_per_patch;
    uint4 *dst = static_cast<uint4 *>(a.h) + (size_t)g * total;
    for (long v = (long)blockIdx.x * blockDim.x + threadIdx.x; v < total; v += (long)gridDim.x * blockDim.x) {
        const int t = (int)(v / vec_per_patch);
        const int off = (int)(v - (long)t * vec_per_patch);
        dst[v] = src[(size_t)clampi(pid[t], a.m) * vec_per_patch + off];
    }
}

hipError_t launch_gather(const GatherArgs &a, bool bf16, hipStream_t st)
{
    const int l_p = a.l / a.m;
    const int elem = bf16 ? 2 : 4;
    const int vec_per_patch = (int)(((size_t)l_p * a.d * elem) / 16);  // d % 8 == 0 => exact
    const long total = (long)a.c * vec_per_patch;
    long blocks = (total + 256 * 4 - 1) / (256 * 4);  // ~4 vectors per thread
    if (blocks < 1) blocks = 1;
    if (blocks > 65535) blocks = 65535;
    hipLaunchKernelGGL(gather_kernel, dim3((unsigned)blocks, a.b * a.k), dim3(256), 0, st, a, vec_per_patch);
    return hipGetLastError();
}

}  // namespace uoe

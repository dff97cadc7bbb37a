// One translation unit per large-kernel size: compiled with -DESC_KS=<Ks> (0 builds the
// variant without conv items that esc_dynkernel_gen and pure copies use).  Instantiates
// forward_kernel<Ks, RY, T, STAGED> for both register blockings, both storage types and
// both estimator flavours, and exports one host function that launches the one asked for.
#include "esc_kernels.hpp"

#ifndef ESC_KS
#error "compile with -DESC_KS=<kernel size>"
#endif

namespace esc {

#define ESC_CAT2(a, b) a##b
#define ESC_CAT(a, b) ESC_CAT2(a, b)

namespace {

template <int KS, int RY, typename T>
hipError_t launch_flavour(bool staged, unsigned grid, hipStream_t s, const FwdParams &p)
{
    if (staged)
        hipLaunchKernelGGL((forward_kernel<KS, RY, T, true>), dim3(grid), dim3(kThreads), 0, s, p);
    else
        hipLaunchKernelGGL((forward_kernel<KS, RY, T, false>), dim3(grid), dim3(kThreads), 0, s, p);
    return hipGetLastError();
}

template <int KS, int RY, typename T>
hipError_t occupancy_flavour(bool staged, int *blocks_per_cu)
{
    if (staged)
        return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, forward_kernel<KS, RY, T, true>, kThreads, 0);
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, forward_kernel<KS, RY, T, false>, kThreads, 0);
}

}  // namespace

// ry: 2 or 4 (4 exists for Ks <= 17 only; Ks == 0 ignores it)
__attribute__((visibility("hidden"))) hipError_t ESC_CAT(launch_ks_, ESC_KS)(int ry, bool bf16, bool staged,
                                                                             unsigned grid, hipStream_t s,
                                                                             const FwdParams &p)
{
    constexpr int KS = ESC_KS;
    if constexpr (KS > 0 && KS <= 17) {
        if (ry == 4)
            return bf16 ? launch_flavour<KS, 4, bf16_t>(staged, grid, s, p)
                        : launch_flavour<KS, 4, float>(staged, grid, s, p);
    }
    return bf16 ? launch_flavour<KS, 2, bf16_t>(staged, grid, s, p) : launch_flavour<KS, 2, float>(staged, grid, s, p);
}

// resident blocks per compute unit the runtime grants this variant on the current device
__attribute__((visibility("hidden"))) hipError_t ESC_CAT(occupancy_ks_, ESC_KS)(int ry, bool bf16, bool staged,
                                                                                int *blocks_per_cu)
{
    constexpr int KS = ESC_KS;
    if constexpr (KS > 0 && KS <= 17) {
        if (ry == 4)
            return bf16 ? occupancy_flavour<KS, 4, bf16_t>(staged, blocks_per_cu)
                        : occupancy_flavour<KS, 4, float>(staged, blocks_per_cu);
    }
    return bf16 ? occupancy_flavour<KS, 2, bf16_t>(staged, blocks_per_cu)
                : occupancy_flavour<KS, 2, float>(staged, blocks_per_cu);
}

}  // namespace esc

// Interface between the host side (esc_api.hip) and the depth-wise branch of ConvFFN
// (esc_ffn.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace esc {

// v[n, m, y, x] = u[n, m, y, x] + gelu(bk[m] + sum_{i,j<3} k[m*9 + i*3 + j] * u~[n, m, y+i-1, x+j-1]),
// u~ = u extended by zeros; u and v are stacks of `planes` = N * C_h planes of H x W
// elements in the storage type, plane after plane; plane q uses channel q % Ch's kernel.
struct FfnBranchParams {
    const void *u;
    void *v;
    const float *k;   // [Ch, 3, 3]
    const float *bk;  // [Ch] or nullptr
    int Ch, H, W;
    long planes;
};

hipError_t launch_ffn_branch(const FfnBranchParams &p, bool bf16, hipStream_t s);

}  // namespace esc

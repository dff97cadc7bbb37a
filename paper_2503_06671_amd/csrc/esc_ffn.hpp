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

// The whole network in one launch for C <= 64 and Ch <= 128 (neither U nor V
// leaves the chip): out = w2 . V + b2, V = U + gelu(k (*) U + bk), U = gelu(w1 . x + b1).
// Returns hipErrorNotSupported, with nothing launched, for other shapes and for problems of
// too few strips and bands to fill the chip.
struct FfnStreamParams {
    const void *x;         // storage type: fp32, or bf16 bit patterns (bf16 != 0)
    void *out;
    int bf16;
    const float *w1, *b1;  // [Ch, C], [Ch] or nullptr
    const float *k, *bk;   // [Ch, 3, 3], [Ch] or nullptr
    const float *w2, *b2;  // [C, Ch], [C] or nullptr
    int N, C, H, W, Ch;
    int rows_per_band, strips, bands;  // set by launch_ffn_stream
};

hipError_t launch_ffn_stream(const FfnStreamParams &p, hipStream_t s);

}  // namespace esc

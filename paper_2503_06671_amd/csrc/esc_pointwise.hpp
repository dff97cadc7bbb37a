// Interface between the host side (esc_api.hip) and the point-wise convolution kernel
// (esc_pointwise.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace esc {

// dst[n, m, q] = act(bias[m] + sum_k w[m * w_ld + k] * cat[n, k, q]) (+ res[n, m, q]),  m < M, q < P,
// where cat's first K1 channels are src1's and the next K2 are src2's, and act is the
// identity or (gelu != 0) the exact erf GELU.  Every tensor is a
// stack of planes of P elements in the storage type; image n of a tensor starts
// n * <its>_img_stride elements after the base (channel planes follow one another).
struct PointwiseParams {
    const void *src1, *src2;
    size_t src1_img_stride, src2_img_stride;
    int K1, K2;
    const float *w;
    int w_ld;
    const float *bias;  // [M] or nullptr
    const void *res;    // residual or nullptr
    size_t res_img_stride;
    void *dst;
    size_t dst_img_stride;
    int M, N;
    long P;
    int gelu;           // != 0: GELU on the product plus bias (ConvFFN's first layer)
};

constexpr int kPointwiseMaxK = 240;  // input channels the kernel's LDS staging holds

hipError_t launch_pointwise(const PointwiseParams &p, bool bf16, hipStream_t s);

}  // namespace esc

// Interface between the host side (esc_api.hip) and the backward kernels (esc_backward.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace esc {

constexpr int kCorrTileW = 64, kCorrTileH = 32;  // pixels per block of the correlation kernel

// the correlation window: Ks x Ks, or 3 x 3 when Ks == 1 (DK's gradient is its centre 3 x 3)
__host__ __device__ inline int corr_window(int Ks) { return Ks < 3 ? 3 : Ks; }
__host__ __device__ inline int corr_tiles(int H, int W)
{
    return ((W + kCorrTileW - 1) / kCorrTileW) * ((H + kCorrTileH - 1) / kCorrTileH);
}
// floats of per-tile partial sums: per (image, channel, tile) the window's Kc*Kc sums and the sum of x
inline size_t corr_partial_floats(int N, int Ca, int H, int W, int Ks)
{
    const size_t kc = (size_t)corr_window(Ks);
    return (size_t)N * Ca * corr_tiles(H, W) * (kc * kc + 1);
}

struct BackwardParams {
    const void *x, *go;      // [N,C,H,W] storage type
    int N, C, Ca, H, W, Ks;
    const float *lk;         // forward's large kernel
    long lk_cstride;
    int hidden;              // estimator (has_gen != 0), as in the forward
    int has_gen;
    const float *w_down, *b_down, *w_up, *b_up;
    const float *dk_in;      // DK given by the caller (has_gen == 0), or nullptr (DK = 0)
    // workspace pieces (fp32)
    float *partial;          // corr_partial_floats
    float *ddk;              // [N,Ca,9]   dL/dDK
    float *g;                // [N,Ca]     GAP means
    float *t;                // [N,K]      estimator's hidden activations (or g)
    float *du;               // [N,hidden] dL/du
    float *dgc;              // [N,Ca]     dL/dg / (H W): the constant added to dx's planes
    float *dkf;              // [N,Ca,9]   DK, flipped (the kernel of the input gradient)
    float *lkf;              // [Ca,Ks,Ks] LK, flipped (dense, channel stride Ks*Ks; one filter when lk_cstride == 0)
    // caller's gradient buffers (any may be nullptr)
    float *grad_lk, *grad_dk, *grad_w_down, *grad_b_down, *grad_w_up, *grad_b_up;
    int accumulate;          // parameter gradients are added to what the buffers hold
    int corr_vec;            // set by launch_backward_sums: the correlation fetches its tiles in 16-byte pieces
};

// 1. correlation of grad_out with x per tile (partial sums in the workspace)
hipError_t launch_backward_sums(const BackwardParams &p, bool bf16, hipStream_t s);
// 2. per image: dDK and g from the tiles' sums, the estimator forwards (DK) and backwards
//    (dL/dg), the flipped kernels - all that the input gradient's launch needs
hipError_t launch_backward_estimator(const BackwardParams &p, hipStream_t s);
// 3. the sums over the batch: grad_lk and the estimator's parameter gradients
hipError_t launch_backward_batch_sums(const BackwardParams &p, hipStream_t s);

}  // namespace esc

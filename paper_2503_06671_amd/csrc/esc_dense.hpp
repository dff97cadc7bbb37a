// Interface between the host side (esc_api.hip) and the dense large-kernel convolution
// kernels (esc_dense.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace esc {

constexpr int kDenseMaxCa = 64;   // attention channels the dense form handles (four tiles of 16)
constexpr int kDenseMaxKs = 17;   // largest dense kernel (its halo tile and weight rows must fit in LDS)

struct DenseParams {
    const void *x;      // [N,C,H,W] storage type
    void *out;          // [N,C,H,W] storage type
    const float *wt;    // weights rearranged by launch_dense_weights (workspace)
    const float *dk;    // [N,Ca,3,3] fp32 or nullptr (DK = 0)
    int N, C, Ca, H, W, Ks;
    int tiles_x, tiles_y;
    // pass-through copy: every block moves `copy_share` bytes (a multiple of 4096, or the whole
    // range by elements when copy_vec is 0) of its image's identity range [idt_off, idt_off + idt_len)
    size_t img_bytes, idt_off, idt_len, copy_share;
    int copy_vec, elem_bytes;
    // set by launch_dense: division by the halo tile's width and by its rows x width as a
    // multiply-high and a shift (the tile fill locates every element with both)
    unsigned hc_mul, hc_shift, hp_mul, hp_shift;
    // bf16 matrix path: whether the tile is fetched in 16-byte pieces
    int fill_vec;
};

// the kernel size the device code walks: a 1 x 1 kernel is embedded in a 3 x 3 one
inline int dense_effective_ks(int Ks) { return Ks < 3 ? 3 : Ks; }

// up to 16 channels run on the bf16 matrix instructions: bf16 storage for every kernel size,
// fp32 storage (every value and weight as three exact bf16 terms, three tiles in LDS) up to 13 x 13
inline bool dense_on_bf16_mfma(int Ca, int Ks, bool bf16) { return Ca <= 16 && (bf16 || dense_effective_ks(Ks) <= 13); }

// floats the rearranged weights take: [CT chunks][Kse rows][Kse taps][CT][16 ci][16 co], or, for
// the bf16 matrix path, [(Kse + 1) / 2 pairs of tap columns][Kse rows][2 or 3 terms][64 lanes][8 bf16]
// (the storage type is not known when a workspace is sized: room for three terms)
inline size_t dense_weight_floats(int Ca, int Ks)
{
    const size_t ct = (size_t)(Ca + 15) / 16, kse = (size_t)dense_effective_ks(Ks);
    return ct == 1 ? kse * (kse + 1) * 384 : ct * kse * kse * ct * 256;
}

hipError_t launch_dense_weights(const float *lk, int Ca, int Ks, bool bf16, float *wt, hipStream_t s);
hipError_t launch_dense(const DenseParams &p, bool bf16, hipStream_t s);

}  // namespace esc

// Point-wise (1x1) convolutions of the ConvAttn module for gfx950 (MI355X): Conv_fuse on
// Concat(F_res, F_idt) (Eq. 4 line 4 of the ESC paper), the point-wise large-kernel
// factor LK^c of Eq. 5, and the residual add of Eq. 3 line 3 in the same pass.
//
// A 1x1 convolution in NCHW is the dense contraction  D[M x P] = W[M x K] . B[K x P]
// per image, with P = H*W pixels contiguous in memory for every channel of B and D, so
// it runs on the matrix cores: v_mfma_f32_32x32x2_f32, fp32 products and fp32
// accumulation (bf16 storage is widened exactly on load and rounded once at the store).
// The input channels come from two tensors (the first K1 from `src1`, the other K2 from
// `src2`): that is the concat, which is never materialised.
//
// One wavefront owns 32*Q consecutive pixels and, 64 output channels at a time, all of
// their outputs: accumulators 2 x Q tiles of 32 x 32.  The weights of the 64 channels are
// staged transposed in LDS (w_t[k][m], so that the A operand - lane l holds
// W[m = l % 32][k = l / 32] - is a conflict-free read); the B operand - lane l holds
// B[k = l / 32][pixel l % 32] - comes straight from global memory, Q pixels per lane and
// channel in one access, eight channel pairs in flight while the previous eight are
// multiplied.  Pixel j of MFMA tile q is pixel Q*j + q of the wavefront's run, so a lane's
// Q results for one output channel are neighbours in memory and leave in one store.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "esc_pointwise.hpp"

namespace esc {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kPwThreads = 256;
constexpr int kPwChunkM = 64;  // output channels per pass over the inputs
constexpr int kPwBatch = 8;    // channel pairs whose loads are in flight together
constexpr int kPwPitch = kPwChunkM + 1;  // floats between two rows of the staged weights (odd: no bank conflicts)

struct bf16s {
    uint16_t bits;
};

__device__ __forceinline__ uint16_t pw_f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Q consecutive elements from p (aligned to all Q when VEC), widened to fp32
template <typename T, int Q, bool VEC, bool NT>
__device__ __forceinline__ void load_q(const T *p, float (&v)[Q])
{
    if constexpr (std::is_same<T, float>::value) {
        if constexpr (VEC && Q == 2) {
            const f32x2 t = NT ? __builtin_nontemporal_load(reinterpret_cast<const f32x2 *>(p))
                               : *reinterpret_cast<const f32x2 *>(p);
            v[0] = t.x;
            v[1] = t.y;
        } else {
#pragma unroll
            for (int q = 0; q < Q; ++q) v[q] = NT ? __builtin_nontemporal_load(p + q) : p[q];
        }
    } else {
        if constexpr (VEC && Q == 2) {
            const uint32_t w = NT ? __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(p))
                                  : *reinterpret_cast<const uint32_t *>(p);
            v[0] = __uint_as_float(w << 16);
            v[1] = __uint_as_float(w & 0xffff0000u);
        } else {
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const uint16_t b = NT ? __builtin_nontemporal_load(&p[q].bits) : p[q].bits;
                v[q] = __uint_as_float((uint32_t)b << 16);
            }
        }
    }
}

// the first `cnt` of Q consecutive results to p (all Q in one access when VEC; cnt == Q then)
template <typename T, int Q, bool VEC>
__device__ __forceinline__ void store_q(T *p, const float (&v)[Q], int cnt)
{
    if constexpr (std::is_same<T, float>::value) {
        if constexpr (VEC && Q == 2) {
            const f32x2 t = {v[0], v[1]};
            __builtin_nontemporal_store(t, reinterpret_cast<f32x2 *>(p));
        } else {
#pragma unroll
            for (int q = 0; q < Q; ++q)
                if (q < cnt) __builtin_nontemporal_store(v[q], p + q);
        }
    } else {
        if constexpr (VEC && Q == 2) {
            const uint32_t w = (uint32_t)pw_f32_to_bf16(v[0]) | ((uint32_t)pw_f32_to_bf16(v[1]) << 16);
            __builtin_nontemporal_store(w, reinterpret_cast<uint32_t *>(p));
        } else {
#pragma unroll
            for (int q = 0; q < Q; ++q)
                if (q < cnt) __builtin_nontemporal_store(pw_f32_to_bf16(v[q]), &p[q].bits);
        }
    }
}

extern __shared__ __align__(16) float pw_lds[];  // w_t[k][kPwPitch]: the pass's weights, transposed

template <typename T, int Q, bool VEC>
__global__ __launch_bounds__(kPwThreads) void pointwise_kernel(const PointwiseParams p)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int K = p.K1 + p.K2, Kp = (K + 1) & ~1;
    const long P = p.P;
    constexpr int kTilePx = (kPwThreads / 64) * 32 * Q;  // pixels per block
    const unsigned tiles = (unsigned)((P + kTilePx - 1) / kTilePx);
    const unsigned n = blockIdx.x / tiles, tile = blockIdx.x - n * tiles;
    // this lane's Q pixels: px .. px + Q - 1 of image n; what lies beyond the image is
    // loaded from clamped addresses (its columns of the product are never stored)
    const long px = (long)tile * kTilePx + wave * 32 * Q + l32 * Q;
    const long px_ld = VEC ? (px < P ? px : P - Q) : px;
    const int n_valid = px >= P ? 0 : (P - px < Q ? (int)(P - px) : Q);

    const T *s1 = (const T *)p.src1 + (size_t)n * p.src1_img_stride;
    const T *s2 = (const T *)p.src2 + (size_t)n * p.src2_img_stride;
    auto load_b = [&](int kk, float (&v)[Q]) {  // channel 2*kk + half of the concat
        int k = 2 * kk + half;
        k = k < K ? k : K - 1;  // (odd K: the pad channel is zeroed below)
        const bool first = k < p.K1;
        const T *plane = first ? s1 + (size_t)k * P : s2 + (size_t)(k - p.K1) * P;
        if constexpr (VEC) {
            if (first)
                load_q<T, Q, VEC, false>(plane + px_ld, v);
            else
                load_q<T, Q, VEC, true>(plane + px_ld, v);
        } else {
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const long e = px + q < P ? px + q : P - 1;
                float one[1];
                load_q<T, 1, false, false>(plane + e, one);
                v[q] = one[0];
            }
        }
        // A pad channel (odd K) multiplies a zero weight: its value must be finite.
        if (2 * kk + half >= K) {
#pragma unroll
            for (int q = 0; q < Q; ++q) v[q] = 0.f;
        }
    };

    for (int m0 = 0; m0 < p.M; m0 += kPwChunkM) {
        // ---- stage w_t[k][m] = W[m0 + m][k] (zero beyond M and beyond K) ----
        __syncthreads();  // the previous pass has finished with the staging area
        for (int idx = threadIdx.x; idx < Kp * kPwChunkM; idx += kPwThreads) {
            const int m = idx / Kp, k = idx - m * Kp;  // consecutive threads read along a weight row
            float w = 0.f;
            if (m0 + m < p.M && k < K) w = p.w[(size_t)(m0 + m) * p.w_ld + k];
            pw_lds[k * kPwPitch + m] = w;
        }
        __syncthreads();
        const bool two = m0 + 32 < p.M;  // the pass has a second tile of 32 output channels

        // ---- accumulators start from the bias ----
        f32x16 acc[2][Q];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int co = m0 + 32 * mt + 8 * (r >> 2) + 4 * half + (r & 3);
                const float b = (p.bias != nullptr && co < p.M) ? p.bias[co] : 0.f;
#pragma unroll
                for (int q = 0; q < Q; ++q) acc[mt][q][r] = b;
            }

        // ---- the contraction, kPwBatch channel pairs per round, the next round's loads in flight ----
        const int pairs = Kp / 2;
        float cur[kPwBatch][Q], nxt[kPwBatch][Q];
#pragma unroll
        for (int u = 0; u < kPwBatch; ++u) load_b(u < pairs ? u : pairs - 1, cur[u]);
        for (int kk0 = 0; kk0 < pairs; kk0 += kPwBatch) {
            if (kk0 + kPwBatch < pairs) {
#pragma unroll
                for (int u = 0; u < kPwBatch; ++u) {
                    const int kk = kk0 + kPwBatch + u;
                    load_b(kk < pairs ? kk : pairs - 1, nxt[u]);
                }
            }
#pragma unroll
            for (int u = 0; u < kPwBatch; ++u) {
                const int kk = kk0 + u;
                if (kk < pairs) {  // block-uniform
                    const float a0 = pw_lds[(2 * kk + half) * kPwPitch + l32];
#pragma unroll
                    for (int q = 0; q < Q; ++q)
                        acc[0][q] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, cur[u][q], acc[0][q], 0, 0, 0);
                    if (two) {
                        const float a1 = pw_lds[(2 * kk + half) * kPwPitch + 32 + l32];
#pragma unroll
                        for (int q = 0; q < Q; ++q)
                            acc[1][q] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, cur[u][q], acc[1][q], 0, 0, 0);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < kPwBatch; ++u)
#pragma unroll
                for (int q = 0; q < Q; ++q) cur[u][q] = nxt[u][q];
        }

        // ---- residual (Eq. 3 line 3) and store ----
        T *dn = (T *)p.dst + (size_t)n * p.dst_img_stride;
        const T *rn = p.res != nullptr ? (const T *)p.res + (size_t)n * p.res_img_stride : nullptr;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            if (mt == 1 && !two) break;
            float rv[16][Q];
            if (rn != nullptr) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int co = m0 + 32 * mt + 8 * (r >> 2) + 4 * half + (r & 3);
                    const int cc = co < p.M ? co : p.M - 1;
                    if constexpr (VEC) {
                        load_q<T, Q, VEC, true>(rn + (size_t)cc * P + px_ld, rv[r]);
                    } else {
#pragma unroll
                        for (int q = 0; q < Q; ++q) {
                            const long e = px + q < P ? px + q : P - 1;
                            float one[1];
                            load_q<T, 1, false, true>(rn + (size_t)cc * P + e, one);
                            rv[r][q] = one[0];
                        }
                    }
                }
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int co = m0 + 32 * mt + 8 * (r >> 2) + 4 * half + (r & 3);
                float v[Q];
#pragma unroll
                for (int q = 0; q < Q; ++q) v[q] = acc[mt][q][r] + (rn != nullptr ? rv[r][q] : 0.f);
                if (co < p.M && n_valid > 0) store_q<T, Q, VEC>(dn + (size_t)co * P + px, v, n_valid);
            }
        }
    }
}

template <typename T, int Q, bool VEC>
hipError_t launch_one(const PointwiseParams &p, unsigned grid, size_t lds, hipStream_t s)
{
    hipLaunchKernelGGL((pointwise_kernel<T, Q, VEC>), dim3(grid), dim3(kPwThreads), lds, s, p);
    return hipGetLastError();
}

}  // namespace

// Host side: picks the pixels per lane (two once that still gives the chip enough blocks)
// and the access width (vector accesses need even planes and aligned bases), and launches.
__attribute__((visibility("hidden"))) hipError_t launch_pointwise(const PointwiseParams &p, bool bf16, hipStream_t s)
{
    if (p.N < 1 || p.P < 1 || p.M < 1 || p.K1 + p.K2 < 1) return hipSuccess;
    const size_t es = bf16 ? 2 : 4;
    const int K = p.K1 + p.K2, Kp = (K + 1) & ~1;
    if (K > kPointwiseMaxK) return hipErrorInvalidValue;
    const size_t lds = (size_t)Kp * kPwPitch * sizeof(float);
    const long blocks2 = (long)p.N * ((p.P + 255) / 256);
    const int q = blocks2 >= 1024 ? 2 : 1;
    auto aligned = [&](const void *ptr, size_t img_stride) {
        return ptr == nullptr || ((uintptr_t)ptr % (2 * es) == 0 && img_stride % 2 == 0);
    };
    const bool vec = q == 2 && p.P % 2 == 0 && aligned(p.src1, p.src1_img_stride) && aligned(p.src2, p.src2_img_stride) &&
                     aligned(p.res, p.res_img_stride) && aligned(p.dst, p.dst_img_stride);
    const long tile_px = 4L * 32 * q;
    const long grid = (long)p.N * ((p.P + tile_px - 1) / tile_px);
    if (grid >= (1L << 31)) return hipErrorInvalidValue;
    if (q == 1)
        return bf16 ? launch_one<bf16s, 1, false>(p, (unsigned)grid, lds, s) : launch_one<float, 1, false>(p, (unsigned)grid, lds, s);
    if (vec) return bf16 ? launch_one<bf16s, 2, true>(p, (unsigned)grid, lds, s) : launch_one<float, 2, true>(p, (unsigned)grid, lds, s);
    return bf16 ? launch_one<bf16s, 2, false>(p, (unsigned)grid, lds, s) : launch_one<float, 2, false>(p, (unsigned)grid, lds, s);
}

}  // namespace esc

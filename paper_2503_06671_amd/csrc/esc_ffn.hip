// The depth-wise branch of ConvFFN for gfx950 (MI355X): between the two point-wise layers
// of the feed-forward network that precedes every ConvAttn module (Eq. 3 line 3 of the ESC
// paper; Sec. 3 fixes the kernel size at three),
//
//     V = U + gelu(K (*) U + bk),      K depth-wise 3 x 3, zero padding, erf-form GELU.
//
// Nine multiply-adds and one GELU per element on 2 x 4 (or 2 x 2) bytes of traffic: bound by
// HBM, so the kernel is laid out for coalesced 16-byte accesses and nothing else.  A thread
// owns a column strip one 16-byte piece wide and kRows rows high of one plane: it walks down
// the strip with the rows above and below in registers, so every row of the strip is
// fetched once per thread (its left and right neighbours' elements come from the
// neighbouring pieces' cache lines).  Neighbouring lanes own neighbouring pieces of a row.
// fp32 arithmetic; bf16 storage is widened exactly and rounded once at the store.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "esc_ffn.hpp"

namespace esc {
namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int kFbThreads = 256;
constexpr int kFbRows = 4;  // rows of a thread's strip

// GELU of ConvFFN, v * Phi(v) with the erf of Phi evaluated by the rational approximation
// 7.1.26 of Abramowitz and Stegun's handbook (|error| <= 1.5e-7 in erf, i.e. <= 1e-7 |v| in the
// result: a hundredth of the fp32 parity bar): erf(a) = 1 - (a1 t + ... + a5 t^5) exp(-a^2),
// t = 1 / (1 + p a), a = |v| / sqrt(2).  A reciprocal, an exponential and a dozen multiply-adds,
// no branch - a third of the library erf's instructions, which at one GELU per hidden element
// twice over were most of the vector units' time in these kernels.
__device__ __forceinline__ float fb_gelu(float v)
{
    const float a = fabsf(v) * 0.70710678118654752440f;
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, a, 1.f));
    float q = fmaf(1.061405429f, t, -1.453152027f);
    q = fmaf(q, t, 1.421413741f);
    q = fmaf(q, t, -0.284496736f);
    q = fmaf(q, t, 0.254829592f);
    const float e = __builtin_amdgcn_exp2f(a * a * -1.44269504088896340736f);
    const float erf_a = fmaf(-q * t, e, 1.f);          // erf(|v| / sqrt 2) >= 0
    const float h = 0.5f * v;
    return fmaf(fabsf(h), erf_a, h);                   // 0.5 v (1 + sign(v) erf_a)
}

__device__ __forceinline__ uint16_t fb_f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <typename T>
__device__ __forceinline__ float fb_load1(const T *p)
{
    if constexpr (sizeof(T) == 4)
        return *p;
    else
        return __uint_as_float((uint32_t)*p << 16);
}

// One row of a strip, widened: e[0] is the element left of the piece, e[1 .. PER] the
// piece, e[PER + 1] the element right of it; zeros outside the image.
template <typename T, int PER, bool VEC>
__device__ __forceinline__ void fb_row(const T *plane, int y, int x0, int H, int W, float (&e)[PER + 2])
{
    const bool row_in = y >= 0 && y < H;
    const int yc = y < 0 ? 0 : (y >= H ? H - 1 : y);
    const T *row = plane + (size_t)yc * W;
    if constexpr (VEC) {
        // W % PER == 0 and an aligned base: the piece is inside the row as a whole
        const u32x4 r = *reinterpret_cast<const u32x4 *>(row + x0);
        const float l = fb_load1(row + (x0 > 0 ? x0 - 1 : 0));
        const float rr = fb_load1(row + (x0 + PER < W ? x0 + PER : W - 1));
        if constexpr (sizeof(T) == 4) {
            e[1] = __uint_as_float(r.x), e[2] = __uint_as_float(r.y), e[3] = __uint_as_float(r.z), e[4] = __uint_as_float(r.w);
        } else {
            e[1] = __uint_as_float(r.x << 16), e[2] = __uint_as_float(r.x & 0xffff0000u);
            e[3] = __uint_as_float(r.y << 16), e[4] = __uint_as_float(r.y & 0xffff0000u);
            e[5] = __uint_as_float(r.z << 16), e[6] = __uint_as_float(r.z & 0xffff0000u);
            e[7] = __uint_as_float(r.w << 16), e[8] = __uint_as_float(r.w & 0xffff0000u);
        }
        e[0] = x0 > 0 ? l : 0.f;
        e[PER + 1] = x0 + PER < W ? rr : 0.f;
    } else {
#pragma unroll
        for (int j = 0; j < PER + 2; ++j) {
            const int x = x0 - 1 + j;
            const float v = fb_load1(row + (x < 0 ? 0 : (x >= W ? W - 1 : x)));
            e[j] = (x >= 0 && x < W) ? v : 0.f;
        }
    }
    if (!row_in) {
#pragma unroll
        for (int j = 0; j < PER + 2; ++j) e[j] = 0.f;
    }
}

template <typename T, bool VEC>
__global__ __launch_bounds__(kFbThreads) void ffn_branch_kernel(const FfnBranchParams p)
{
    constexpr int PER = VEC ? 16 / (int)sizeof(T) : 1;
    const int pieces = (p.W + PER - 1) / PER;           // per row
    const int strips = (p.H + kFbRows - 1) / kFbRows;   // per piece column
    const long per_plane = (long)pieces * strips;
    const long total = per_plane * p.planes;
    for (long idx = (long)blockIdx.x * kFbThreads + threadIdx.x; idx < total; idx += (long)gridDim.x * kFbThreads) {
        const long plane_i = idx / per_plane;
        const int rem = (int)(idx - plane_i * per_plane);
        const int sy = rem / pieces, x0 = (rem - sy * pieces) * PER, y0 = sy * kFbRows;
        const int ch = (int)(plane_i % p.Ch);
        const T *up = (const T *)p.u + (size_t)plane_i * p.H * p.W;
        T *vp = (T *)p.v + (size_t)plane_i * p.H * p.W;
        float k[9];
#pragma unroll
        for (int t = 0; t < 9; ++t) k[t] = p.k[(size_t)ch * 9 + t];
        const float b = p.bk != nullptr ? p.bk[ch] : 0.f;

        float ra[PER + 2], rb[PER + 2], rc[PER + 2];
        fb_row<T, PER, VEC>(up, y0 - 1, x0, p.H, p.W, ra);
        fb_row<T, PER, VEC>(up, y0, x0, p.H, p.W, rb);
#pragma unroll
        for (int r = 0; r < kFbRows; ++r) {
            const int y = y0 + r;
            if (y >= p.H) break;
            fb_row<T, PER, VEC>(up, y + 1, x0, p.H, p.W, rc);
            float o[PER];
#pragma unroll
            for (int j = 0; j < PER; ++j) {
                float s = b;
                s = fmaf(k[0], ra[j], s), s = fmaf(k[1], ra[j + 1], s), s = fmaf(k[2], ra[j + 2], s);
                s = fmaf(k[3], rb[j], s), s = fmaf(k[4], rb[j + 1], s), s = fmaf(k[5], rb[j + 2], s);
                s = fmaf(k[6], rc[j], s), s = fmaf(k[7], rc[j + 1], s), s = fmaf(k[8], rc[j + 2], s);
                o[j] = rb[j + 1] + fb_gelu(s);
            }
            T *dst = vp + (size_t)y * p.W + x0;
            if constexpr (VEC) {
                u32x4 w;
                if constexpr (sizeof(T) == 4) {
                    w = u32x4{__float_as_uint(o[0]), __float_as_uint(o[1]), __float_as_uint(o[2]), __float_as_uint(o[3])};
                } else {
                    w = u32x4{(uint32_t)fb_f32_to_bf16(o[0]) | ((uint32_t)fb_f32_to_bf16(o[1]) << 16),
                              (uint32_t)fb_f32_to_bf16(o[2]) | ((uint32_t)fb_f32_to_bf16(o[3]) << 16),
                              (uint32_t)fb_f32_to_bf16(o[4]) | ((uint32_t)fb_f32_to_bf16(o[5]) << 16),
                              (uint32_t)fb_f32_to_bf16(o[6]) | ((uint32_t)fb_f32_to_bf16(o[7]) << 16)};
                }
                *reinterpret_cast<u32x4 *>(dst) = w;
            } else {
                if constexpr (sizeof(T) == 4)
                    *dst = o[0];
                else
                    *dst = fb_f32_to_bf16(o[0]);
            }
#pragma unroll
            for (int j = 0; j < PER + 2; ++j) ra[j] = rb[j], rb[j] = rc[j];
        }
    }
}

}  // namespace

__attribute__((visibility("hidden"))) hipError_t launch_ffn_branch(const FfnBranchParams &p, bool bf16, hipStream_t s)
{
    if (p.planes < 1 || p.H < 1 || p.W < 1 || p.Ch < 1) return hipSuccess;
    const int per = bf16 ? 8 : 4;
    const bool vec = p.W % per == 0 && (uintptr_t)p.u % 16 == 0 && (uintptr_t)p.v % 16 == 0;
    const long pieces = vec ? p.W / per : p.W;
    const long strips = (p.H + kFbRows - 1) / kFbRows;
    const long total = pieces * strips * p.planes;
    long grid = (total + kFbThreads - 1) / kFbThreads;
    if (grid > 256L * 32) grid = 256L * 32;  // the blocks loop
    if (vec) {
        if (bf16)
            hipLaunchKernelGGL((ffn_branch_kernel<uint16_t, true>), dim3((unsigned)grid), dim3(kFbThreads), 0, s, p);
        else
            hipLaunchKernelGGL((ffn_branch_kernel<float, true>), dim3((unsigned)grid), dim3(kFbThreads), 0, s, p);
    } else {
        if (bf16)
            hipLaunchKernelGGL((ffn_branch_kernel<uint16_t, false>), dim3((unsigned)grid), dim3(kFbThreads), 0, s, p);
        else
            hipLaunchKernelGGL((ffn_branch_kernel<float, false>), dim3((unsigned)grid), dim3(kFbThreads), 0, s, p);
    }
    return hipGetLastError();
}

}  // namespace esc

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
// A block owns tiles of 128 pixels and, 64 output channels at a time, all of their outputs.
// The input channels pass through LDS in stages of 32, fetched with coalesced 16-byte
// accesses while the stage before is multiplied; the weights of the 64 channels are staged
// once per block, transposed, so that both MFMA operands are conflict-free LDS reads.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "esc_pointwise.hpp"

namespace esc {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int kPwThreads = 256;
constexpr int kPwM = 64;        // output channels per pass over the inputs
constexpr int kPwTile = 128;    // pixels per tile
constexpr int kPwKc = 32;       // input channels per stage
constexpr int kPwWPitch = kPwM + 1;     // floats between two rows of the staged weights (odd: no bank conflicts)
constexpr int kPwBPitch = kPwTile + 4;  // floats between two channel rows of a staged input tile
constexpr int kPwStageW = 8;    // weights a thread fetches together when a pass is staged

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

__device__ __forceinline__ float pw_load1(const float *p) { return *p; }
__device__ __forceinline__ float pw_load1(const bf16s *p) { return __uint_as_float((uint32_t)p->bits << 16); }

typedef __amdgpu_buffer_rsrc_t Rsrc;
constexpr int kRawBuffer = 0x00020000;     // raw buffer (no stride, no swizzle), 32-bit data format
constexpr int kNt = 2;                     // non-temporal
constexpr unsigned kBeyond = 0x80000000u;  // an offset beyond every resource (an image of a tensor is < 2 GiB)

extern __shared__ __align__(16) float pw_lds[];

// The kernel: D[M x P] = W[M x K] . B[K x P] + bias (+ residual) per image, B's channels
// coming from two tensors.  A block owns tiles of 128 pixels (tile b, b + grid, ...); per
// tile the K input channels pass through LDS in stages of 32: every thread fetches 16-byte
// pieces of the next stage (fully coalesced: a channel's 128 pixels are one run of memory)
// while the current stage is multiplied, two buffers taking turns, one barrier per stage.
// Wavefront w multiplies output channels 32*(w & 1) .. +31 with pixels 64*(w >> 1) .. +63
// of the tile: two 32 x 32 accumulator tiles, operands read from LDS in the layout
// v_mfma_f32_32x32x2_f32 wants (A: lane l holds W[m = l % 32][k = l / 32], B: lane l holds
// B[k = l / 32][pixel l % 32]).  The weights of the pass (64 output channels) are staged
// once per block, transposed, with the pass's biases behind them.
//
// Loads and what is done with them are kept apart (all of a stage's loads first, their
// uses a stage later): a value touched right after its load would make the compiler wait
// for that load before it issues the next.
template <typename T, bool VEC>
__global__ __launch_bounds__(kPwThreads, (VEC && sizeof(T) == 4) ? 3 : 2) void pointwise_kernel(const PointwiseParams p)
{
    constexpr int kPer = 16 / (int)sizeof(T);               // pixels per 16-byte piece
    constexpr int kPieces = kPwTile / kPer;                  // pieces per channel row of a tile
    constexpr int kRowsPerSweep = kPwThreads / kPieces;      // channel rows the block fetches at once
    constexpr int kLoads = kPwKc / kRowsPerSweep;            // pieces per thread and stage
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int mt = wave & 1, ph = wave >> 1;
    const int K = p.K1 + p.K2;
    const int stages = (K + kPwKc - 1) / kPwKc;              // per tile
    const int Kr = stages * kPwKc;
    const long P = p.P;
    const unsigned tiles_per_img = (unsigned)((P + kPwTile - 1) / kPwTile);
    const unsigned n_tiles = tiles_per_img * (unsigned)p.N;

    float *s_w = pw_lds;                          // [Kr][kPwWPitch]
    float *s_bias = s_w + Kr * kPwWPitch;         // [kPwM]
    float *s_b = s_bias + kPwM;                   // [2][kPwKc][kPwBPitch]

    // this thread's pieces of a stage: channel row my_row + u * kRowsPerSweep, pixels my_px ..
    const int my_row = tid / kPieces, my_px = (tid - my_row * kPieces) * kPer;

    // fetch: stage `st` of tile `tile` into registers (raw storage bits)
    auto fetch = [&](unsigned tile, int st, u32x4 (&r)[kLoads]) {
        const unsigned n = tile / tiles_per_img;
        const long px0 = (long)(tile - n * tiles_per_img) * kPwTile + my_px;
        const T *s1 = (const T *)p.src1 + (size_t)n * p.src1_img_stride;
        const T *s2 = (const T *)p.src2 + (size_t)n * p.src2_img_stride;
#pragma unroll
        for (int u = 0; u < kLoads; ++u) {
            int k = st * kPwKc + my_row + u * kRowsPerSweep;
            k = k < K ? k : K - 1;  // (rows beyond K are zeroed when they are staged)
            const T *plane = k < p.K1 ? s1 + (size_t)k * P : s2 + (size_t)(k - p.K1) * P;
            if constexpr (VEC) {
                const long e = px0 < P ? px0 : P - kPer;  // P % kPer == 0: a piece is inside or outside as a whole
                r[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(plane + e));
            } else {
                float v[kPer];
#pragma unroll
                for (int e = 0; e < kPer; ++e) v[e] = pw_load1(plane + (px0 + e < P ? px0 + e : P - 1));
                if constexpr (sizeof(T) == 4) {
                    r[u] = u32x4{__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
                } else {
                    r[u] = u32x4{(__float_as_uint(v[0]) >> 16) | (__float_as_uint(v[1]) & 0xffff0000u),
                                 (__float_as_uint(v[2]) >> 16) | (__float_as_uint(v[3]) & 0xffff0000u),
                                 (__float_as_uint(v[4]) >> 16) | (__float_as_uint(v[5]) & 0xffff0000u),
                                 (__float_as_uint(v[6]) >> 16) | (__float_as_uint(v[7]) & 0xffff0000u)};
                }
            }
        }
    };
    // stage: the fetched pieces, widened to fp32, into buffer `buf`; rows beyond K as zeros
    // (their weights are zero too, but zero times a stray Inf would not be)
    auto stage = [&](int st, const u32x4 (&r)[kLoads], int buf) {
        float *dst = s_b + buf * (kPwKc * kPwBPitch);
#pragma unroll
        for (int u = 0; u < kLoads; ++u) {
            const int row = my_row + u * kRowsPerSweep;
            const bool live = st * kPwKc + row < K;
            float *d = dst + row * kPwBPitch + my_px;
            if constexpr (sizeof(T) == 4) {
                const f32x4 v = {__uint_as_float(r[u].x), __uint_as_float(r[u].y), __uint_as_float(r[u].z), __uint_as_float(r[u].w)};
                *reinterpret_cast<f32x4 *>(d) = live ? v : f32x4{0.f, 0.f, 0.f, 0.f};
            } else {
                const f32x4 lo = {__uint_as_float(r[u].x << 16), __uint_as_float(r[u].x & 0xffff0000u),
                                  __uint_as_float(r[u].y << 16), __uint_as_float(r[u].y & 0xffff0000u)};
                const f32x4 hi = {__uint_as_float(r[u].z << 16), __uint_as_float(r[u].z & 0xffff0000u),
                                  __uint_as_float(r[u].w << 16), __uint_as_float(r[u].w & 0xffff0000u)};
                *reinterpret_cast<f32x4 *>(d) = live ? lo : f32x4{0.f, 0.f, 0.f, 0.f};
                *reinterpret_cast<f32x4 *>(d + 4) = live ? hi : f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
    };

    u32x4 regs[kLoads];
    if (blockIdx.x < n_tiles) fetch(blockIdx.x, 0, regs);  // the first inputs are asked for before the weights are staged

    for (int m0 = 0; m0 < p.M; m0 += kPwM) {
        // ---- the pass's weights, transposed: s_w[k][m] = W[m0 + m][k], zero beyond M and K;
        // sixteen consecutive threads read sixteen consecutive weights of a row ----
        __syncthreads();  // every wavefront has finished the previous pass
        for (int i0 = 0; i0 < Kr * kPwM; i0 += kPwStageW * kPwThreads) {
            float wv[kPwStageW];
            bool in[kPwStageW];
#pragma unroll
            for (int u = 0; u < kPwStageW; ++u) {
                const int idx = i0 + u * kPwThreads + tid;
                const int m = (idx >> 4) & (kPwM - 1), k = ((idx >> 10) << 4) + (idx & 15);
                in[u] = m0 + m < p.M && k < K;
                wv[u] = p.w[in[u] ? (size_t)(m0 + m) * p.w_ld + k : 0];
            }
#pragma unroll
            for (int u = 0; u < kPwStageW; ++u) {
                const int idx = i0 + u * kPwThreads + tid;
                const int m = (idx >> 4) & (kPwM - 1), k = ((idx >> 10) << 4) + (idx & 15);
                if (idx < Kr * kPwM) s_w[k * kPwWPitch + m] = in[u] ? wv[u] : 0.f;
            }
        }
        if (tid < kPwM) s_bias[tid] = (p.bias != nullptr && m0 + tid < p.M) ? p.bias[m0 + tid] : 0.f;
        if (m0 > 0 && blockIdx.x < n_tiles) fetch(blockIdx.x, 0, regs);
        // (the barrier of the first stage below also covers the weights)

        f32x16 acc[2];
        int step = 0;  // stages done by this block in this pass: picks the LDS buffer
        for (unsigned tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
            for (int st = 0; st < stages; ++st, ++step) {
                stage(st, regs, step & 1);
                __syncthreads();
                // the next stage's pieces (this tile's, or the next tile's first) fly while this one is multiplied
                if (st + 1 < stages)
                    fetch(tile, st + 1, regs);
                else if (tile + gridDim.x < n_tiles)
                    fetch(tile + gridDim.x, 0, regs);
                if (st == 0) {  // accumulators start from the bias
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float b = s_bias[32 * mt + 8 * (r >> 2) + 4 * half + (r & 3)];
                        acc[0][r] = b;
                        acc[1][r] = b;
                    }
                }
                const float *wk = s_w + (st * kPwKc + half) * kPwWPitch + 32 * mt + l32;
                const float *bk = s_b + (step & 1) * (kPwKc * kPwBPitch) + half * kPwBPitch + 64 * ph + l32;
#pragma unroll 4
                for (int kp = 0; kp < kPwKc / 2; ++kp) {
                    const float a = wk[2 * kp * kPwWPitch];
                    const float b0 = bk[2 * kp * kPwBPitch], b1 = bk[2 * kp * kPwBPitch + 32];
                    acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b0, acc[0], 0, 0, 0);
                    acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b1, acc[1], 0, 0, 0);
                }
            }
            // ---- residual (Eq. 3 line 3) and store: lane l of accumulator tile t holds output
            // channels 8*(r/4) + 4*(l/32) + r%4 of pixel 64*ph + 32*t + l%32.  Buffer accesses on
            // resources that end with the image: rows beyond M and (their offset pushed beyond
            // every resource) pixels beyond the plane read as zero and are not written; without
            // a residual its resource is empty ----
            const unsigned n = tile / tiles_per_img;
            const unsigned px0 = (tile - n * tiles_per_img) * kPwTile + 64 * ph + l32;
            const unsigned plane_bytes = (unsigned)P * (unsigned)sizeof(T);
            const Rsrc rdst = __builtin_amdgcn_make_buffer_rsrc((void *)((T *)p.dst + (size_t)n * p.dst_img_stride), 0,
                                                                (int)((unsigned)p.M * plane_bytes), kRawBuffer);
            const Rsrc rres = __builtin_amdgcn_make_buffer_rsrc(
                (void *)((const T *)p.res + (size_t)n * p.res_img_stride), 0,
                p.res != nullptr ? (int)((unsigned)p.M * plane_bytes) : 0, kRawBuffer);
            if (m0 + 32 * mt < p.M) {  // wavefront-uniform
#pragma unroll
                for (int t2 = 0; t2 < 2; ++t2) {
                    const unsigned px = px0 + 32 * t2;
                    const unsigned px_off = px < (unsigned)P ? px * (unsigned)sizeof(T) : kBeyond;
                    float rv[16];
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const unsigned co = (unsigned)(m0 + 32 * mt + 8 * (r >> 2) + 4 * half + (r & 3));
                        if constexpr (sizeof(T) == 4)
                            rv[r] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rres, (int)(co * plane_bytes + px_off), 0, kNt));
                        else
                            rv[r] = __uint_as_float((unsigned)__builtin_amdgcn_raw_buffer_load_b16(rres, (int)(co * plane_bytes + px_off), 0, kNt) << 16);
                    }
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const unsigned co = (unsigned)(m0 + 32 * mt + 8 * (r >> 2) + 4 * half + (r & 3));
                        const float v = acc[t2][r] + rv[r];
                        if constexpr (sizeof(T) == 4)
                            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), rdst, (int)(co * plane_bytes + px_off), 0, kNt);
                        else
                            __builtin_amdgcn_raw_buffer_store_b16((unsigned short)pw_f32_to_bf16(v), rdst, (int)(co * plane_bytes + px_off), 0, kNt);
                    }
                }
            }
        }
    }
}

template <typename T, bool VEC>
hipError_t launch_one(const PointwiseParams &p, unsigned grid, size_t lds, hipStream_t s)
{
    static size_t granted = 48 * 1024;  // dynamic LDS a launch may ask for without asking first
    if (lds > granted) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&pointwise_kernel<T, VEC>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        granted = lds;
    }
    hipLaunchKernelGGL((pointwise_kernel<T, VEC>), dim3(grid), dim3(kPwThreads), lds, s, p);
    return hipGetLastError();
}

}  // namespace

// Host side: one block per tile of 128 pixels, at most three per compute unit (they loop);
// 16-byte pieces need planes that are multiples of a piece and aligned bases.
__attribute__((visibility("hidden"))) hipError_t launch_pointwise(const PointwiseParams &p, bool bf16, hipStream_t s)
{
    if (p.N < 1 || p.P < 1 || p.M < 1 || p.K1 + p.K2 < 1) return hipSuccess;
    const size_t es = bf16 ? 2 : 4;
    const int K = p.K1 + p.K2;
    if (K > kPointwiseMaxK) return hipErrorInvalidValue;
    // the stores address an image of a tensor with 32-bit byte offsets below 2 GiB
    if ((size_t)p.M * (size_t)p.P * es >= ((size_t)1 << 31)) return hipErrorInvalidValue;
    const int Kr = (K + kPwKc - 1) / kPwKc * kPwKc;
    const size_t lds = ((size_t)Kr * kPwWPitch + kPwM + 2 * (size_t)kPwKc * kPwBPitch) * sizeof(float);
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return hipErrorInvalidDevice;
        cus = n > 0 ? n : 1;
    }
    const long tiles = (long)p.N * ((p.P + kPwTile - 1) / kPwTile);
    if (tiles >= (1L << 31)) return hipErrorInvalidValue;
    const long grid = tiles < 3L * cus ? tiles : 3L * cus;
    const size_t per = 16 / es;
    auto aligned = [&](const void *ptr, size_t img_stride) { return (uintptr_t)ptr % 16 == 0 && img_stride % per == 0; };
    const bool vec = (size_t)p.P % per == 0 && (p.K1 == 0 || aligned(p.src1, p.src1_img_stride)) &&
                     (p.K2 == 0 || aligned(p.src2, p.src2_img_stride));
    if (vec) return bf16 ? launch_one<bf16s, true>(p, (unsigned)grid, lds, s) : launch_one<float, true>(p, (unsigned)grid, lds, s);
    return bf16 ? launch_one<bf16s, false>(p, (unsigned)grid, lds, s) : launch_one<float, false>(p, (unsigned)grid, lds, s);
}

}  // namespace esc

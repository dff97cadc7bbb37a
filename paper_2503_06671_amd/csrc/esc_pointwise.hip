// Point-wise (1x1) convolutions of the ConvAttn module for gfx950 (MI355X): Conv_fuse on
// Concat(F_res, F_idt) (Eq. 4 line 4 of the ESC paper), the point-wise large-kernel
// factor LK^c of Eq. 5, and the residual add of Eq. 3 line 3 in the same pass.
//
// A 1x1 convolution in NCHW is the dense contraction  D[M x P] = W[M x K] . B[K x P]
// per image, with P = H*W pixels contiguous in memory for every channel of B and D, so
// it runs on the matrix cores.  fp32 storage: v_mfma_f32_32x32x2_f32, fp32 products and
// fp32 accumulation.  bf16 storage: v_mfma_f32_32x32x16_bf16 on the stored bf16 values, with
// every fp32 weight split into two bf16 terms (w = hi + lo to 16 mantissa bits, two
// instructions per operand pair: the products are exact in fp32, the accumulation is fp32,
// the result is rounded once at the store) - sixteen times the fp32 form's rate, which
// with bf16 storage was all such a call lasted.
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

// two fp32 values rounded to nearest even and packed, a in the low half: the hardware's
// packed conversion (v_cvt_pk_bf16_f32), one instruction where the shifts and adds above are a dozen
typedef float pw_f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 pw_bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pw_pack2_bf16(float a, float b)
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(pw_f32x2{a, b}, pw_bf16x2));
}

__device__ __forceinline__ float pw_load1(const float *p) { return *p; }
__device__ __forceinline__ float pw_load1(const bf16s *p) { return __uint_as_float((uint32_t)p->bits << 16); }

// GELU of ConvFFN, v * Phi(v) with the erf of Phi evaluated by the rational approximation
// 7.1.26 of Abramowitz and Stegun's handbook (|error| <= 1.5e-7 in erf, i.e. <= 1e-7 |v| in the
// result: a hundredth of the fp32 parity bar): erf(a) = 1 - (a1 t + ... + a5 t^5) exp(-a^2),
// t = 1 / (1 + p a), a = |v| / sqrt(2).  A reciprocal, an exponential and a dozen multiply-adds,
// no branch - a third of the library erf's instructions, which at one GELU per hidden element
// were a quarter of this kernel's time with bf16 storage.
__device__ __forceinline__ float pw_gelu(float v)
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

typedef __amdgpu_buffer_rsrc_t Rsrc;
constexpr int kRawBuffer = 0x00020000;     // raw buffer (no stride, no swizzle), 32-bit data format
constexpr int kNt = 2;                     // non-temporal
constexpr unsigned kBeyond = 0x80000000u;  // an offset beyond every resource (an image of a tensor is < 2 GiB)

extern __shared__ __align__(16) float pw_lds[];

// Residual (Eq. 3 line 3) and store of a wavefront's two 32 x 32 accumulator tiles: lane l
// of tile t holds output channels m0 + 32 mt + 8*(r/4) + 4*(l/32) + r%4 of pixel
// 64 ph + 32 t + l%32 of the block's tile.  Buffer accesses on resources that end with the
// image: rows beyond M and (their offset pushed beyond every resource) pixels beyond the
// plane read as zero and are not written; without a residual its resource is empty.
template <typename T, bool GELU>
__device__ __forceinline__ void store_tile(const PointwiseParams &p, const f32x16 (&acc)[2], unsigned tile,
                                           unsigned tiles_per_img, int m0, int mt, int ph, int l32, int half)
{
    const long P = p.P;
    const unsigned n = tile / tiles_per_img;
    const unsigned px0 = (tile - n * tiles_per_img) * kPwTile + 64 * ph + l32;
    const unsigned plane_bytes = (unsigned)P * (unsigned)sizeof(T);
    const Rsrc rdst = __builtin_amdgcn_make_buffer_rsrc((void *)((T *)p.dst + (size_t)n * p.dst_img_stride), 0,
                                                        (int)((unsigned)p.M * plane_bytes), kRawBuffer);
    const Rsrc rres = __builtin_amdgcn_make_buffer_rsrc((void *)((const T *)p.res + (size_t)n * p.res_img_stride), 0,
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
                const float v = (GELU ? pw_gelu(acc[t2][r]) : acc[t2][r]) + rv[r];
                if constexpr (sizeof(T) == 4)
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), rdst, (int)(co * plane_bytes + px_off), 0, kNt);
                else
                    __builtin_amdgcn_raw_buffer_store_b16((unsigned short)pw_f32_to_bf16(v), rdst, (int)(co * plane_bytes + px_off), 0, kNt);
            }
        }
    }
}

// Fetch of a thread's pieces of stage `st` of tile `tile` into registers (raw storage bits):
// channel rows my_row + u * rows_per_sweep of the stage, pixels my_px ... of the tile.
template <typename T, bool VEC, int LOADS>
__device__ __forceinline__ void fetch_stage(const PointwiseParams &p, unsigned tile, unsigned tiles_per_img, int st,
                                            int my_row, int my_px, int rows_per_sweep, u32x4 (&r)[LOADS])
{
    constexpr int kPer = 16 / (int)sizeof(T);
    const long P = p.P;
    const int K = p.K1 + p.K2;
    const unsigned n = tile / tiles_per_img;
    const long px0 = (long)(tile - n * tiles_per_img) * kPwTile + my_px;
    const T *s1 = (const T *)p.src1 + (size_t)n * p.src1_img_stride;
    const T *s2 = (const T *)p.src2 + (size_t)n * p.src2_img_stride;
#pragma unroll
    for (int u = 0; u < LOADS; ++u) {
        int k = st * kPwKc + my_row + u * rows_per_sweep;
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
}

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
template <typename T, bool VEC, bool GELU>
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

    auto fetch = [&](unsigned tile, int st, u32x4 (&r)[kLoads]) {
        fetch_stage<T, VEC, kLoads>(p, tile, tiles_per_img, st, my_row, my_px, kRowsPerSweep, r);
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
            store_tile<T, GELU>(p, acc, tile, tiles_per_img, m0, mt, ph, l32, half);
        }
    }
}

// The same contraction for bf16 storage, on v_mfma_f32_32x32x16_bf16.  The inputs stay
// bf16 in LDS, [channel][pixel] as they are fetched (16-byte pieces, no widening); an
// operand wants eight consecutive channels of one pixel per lane, so the B operands are
// gathered with 16-bit LDS reads (lanes read consecutive pixels: no bank conflicts).  The
// weights of a pass are staged as two bf16 arrays [64][K], hi = bf16(w) and
// lo = bf16(w - hi): A operands are 16-byte reads, and each B operand is multiplied by
// both.  Same tiles, stages and buffers as the fp32 kernel.  With 16-byte accesses (VEC)
// the operands swap roles - pixels are the rows of the product, output channels its columns
// - so that a lane ends up with runs of four neighbouring pixels of one channel: residual
// added, rounded and packed, they pass through a per-wavefront LDS tile [32 channels][64
// pixels] and leave as 16-byte pieces, eight lanes to a 128-byte run of a channel (stored
// straight from the matrix cores' layout they would be 2-byte elements in 64-byte runs).
constexpr int kPwBfBPitch = kPwTile + 8;  // bf16 elements between two channel rows of a staged input tile
constexpr int kPwBfOPitch = 64;           // bf16 elements of a channel row of a wavefront's output tile (no padding:
                                          // the 16-byte piece q of row ch lies at piece q ^ (ch & 7), which spreads the
                                          // rows over the banks; padded rows would cost the third block per compute unit)

template <bool VEC, bool GELU>
__global__ __launch_bounds__(kPwThreads, VEC ? 3 : 2) void pointwise_bf16_kernel(const PointwiseParams p)
{
    typedef bf16s T;
    typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
    constexpr int kPer = 8;                                  // pixels per 16-byte piece
    constexpr int kPieces = kPwTile / kPer;                  // 16 pieces per channel row of a tile
    constexpr int kRowsPerSweep = kPwThreads / kPieces;      // 16 channel rows at once
    constexpr int kLoads = kPwKc / kRowsPerSweep;            // 2 pieces per thread and stage
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int mt = wave & 1, ph = wave >> 1;
    const int K = p.K1 + p.K2;
    const int stages = (K + kPwKc - 1) / kPwKc;
    const int Kr = stages * kPwKc;
    const int wp = Kr + 8;                                   // bf16 elements between two rows of the staged weights
    const unsigned tiles_per_img = (unsigned)((p.P + kPwTile - 1) / kPwTile);
    const unsigned n_tiles = tiles_per_img * (unsigned)p.N;

    float *s_bias = pw_lds;                                                   // [kPwM]
    uint16_t *s_wh = reinterpret_cast<uint16_t *>(pw_lds + kPwM);             // [kPwM][wp]
    uint16_t *s_wl = s_wh + kPwM * wp;                                        // [kPwM][wp]
    uint16_t *s_b = s_wl + kPwM * wp;                                         // [2][kPwKc][kPwBfBPitch]
    uint16_t *s_o = s_b + 2 * kPwKc * kPwBfBPitch + wave * (32 * kPwBfOPitch);  // VEC: [32][kPwBfOPitch] per wavefront

    const int my_row = tid / kPieces, my_px = (tid - my_row * kPieces) * kPer;
    auto fetch = [&](unsigned tile, int st, u32x4 (&r)[kLoads]) {
        fetch_stage<T, VEC, kLoads>(p, tile, tiles_per_img, st, my_row, my_px, kRowsPerSweep, r);
    };
    // the fetched pieces as they are; rows beyond K as zeros (zero weights times a stray Inf would not be zero)
    auto stage = [&](int st, const u32x4 (&r)[kLoads], int buf) {
        uint16_t *dst = s_b + buf * (kPwKc * kPwBfBPitch);
#pragma unroll
        for (int u = 0; u < kLoads; ++u) {
            const int row = my_row + u * kRowsPerSweep;
            const bool live = st * kPwKc + row < K;
            *reinterpret_cast<u32x4 *>(dst + row * kPwBfBPitch + my_px) = live ? r[u] : u32x4{0u, 0u, 0u, 0u};
        }
    };

    // Two stages are in flight per thread (two register sets taking turns): with the matrix
    // time gone, what such a call lasts is how many bytes the chip has asked for at a time.
    struct Pos {
        unsigned tile;
        int st;
    };
    auto next = [&](Pos q) { return q.st + 1 < stages ? Pos{q.tile, q.st + 1} : Pos{q.tile + gridDim.x, 0}; };
    u32x4 regs_a[kLoads], regs_b[kLoads];
    auto prologue = [&]() {
        const Pos q0{blockIdx.x, 0}, q1 = next(q0);
        if (q0.tile < n_tiles) fetch(q0.tile, q0.st, regs_a);
        if (q1.tile < n_tiles) fetch(q1.tile, q1.st, regs_b);
    };
    prologue();

    for (int m0 = 0; m0 < p.M; m0 += kPwM) {
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
                const float w = in[u] ? wv[u] : 0.f;
                const uint16_t hi = pw_f32_to_bf16(w);
                const uint16_t lo = pw_f32_to_bf16(w - __uint_as_float((uint32_t)hi << 16));
                if (idx < Kr * kPwM) {
                    s_wh[m * wp + k] = hi;
                    s_wl[m * wp + k] = lo;
                }
            }
        }
        if (tid < kPwM) s_bias[tid] = (p.bias != nullptr && m0 + tid < p.M) ? p.bias[m0 + tid] : 0.f;
        if (m0 > 0) prologue();

        f32x16 acc[2];
        int step = 0;  // stages done by this block in this pass: picks the LDS buffer and the register set
        Pos cur{blockIdx.x, 0}, ahead = next(next(cur));
        // one stage: its pieces into LDS, the stage after next asked for into the registers
        // they came from, the products, and behind a tile's last stage its results
        auto body = [&](u32x4 (&regs)[kLoads]) {
            const unsigned tile = cur.tile;
            const int st = cur.st;
            {
                stage(st, regs, step & 1);
                __syncthreads();
                if (ahead.tile < n_tiles) fetch(ahead.tile, ahead.st, regs);
                if (st == 0) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float b = s_bias[VEC ? 32 * mt + l32 : 32 * mt + 8 * (r >> 2) + 4 * half + (r & 3)];
                        acc[0][r] = b;
                        acc[1][r] = b;
                    }
                }
                // weights: lane l holds W[m = l % 32][k = 8 (l / 32) ... + 7] of the 16 channels of a chunk;
                // inputs: lane l holds the same eight channels of pixel l % 32
                const uint16_t *wh = s_wh + (32 * mt + l32) * wp + st * kPwKc + 8 * half;
                const uint16_t *wl = s_wl + (32 * mt + l32) * wp + st * kPwKc + 8 * half;
                const uint16_t *bk = s_b + (step & 1) * (kPwKc * kPwBfBPitch) + (8 * half) * kPwBfBPitch + 64 * ph + l32;
#pragma unroll
                for (int c = 0; c < kPwKc / 16; ++c) {
                    const u32x4 ah = *reinterpret_cast<const u32x4 *>(wh + 16 * c);
                    const u32x4 al = *reinterpret_cast<const u32x4 *>(wl + 16 * c);
                    u32x4 b[2];
#pragma unroll
                    for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
                        for (int w2 = 0; w2 < 4; ++w2) {
                            const uint32_t e0 = bk[(16 * c + 2 * w2) * kPwBfBPitch + 32 * t2];
                            const uint32_t e1 = bk[(16 * c + 2 * w2 + 1) * kPwBfBPitch + 32 * t2];
                            b[t2][w2] = e0 | (e1 << 16);
                        }
#pragma unroll
                    for (int t2 = 0; t2 < 2; ++t2) {
                        if constexpr (VEC) {  // rows = pixels, columns = output channels
                            acc[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, b[t2]),
                                                                              __builtin_bit_cast(bf16x8, ah), acc[t2], 0, 0, 0);
                            acc[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, b[t2]),
                                                                              __builtin_bit_cast(bf16x8, al), acc[t2], 0, 0, 0);
                        } else {
                            acc[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ah),
                                                                              __builtin_bit_cast(bf16x8, b[t2]), acc[t2], 0, 0, 0);
                            acc[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, al),
                                                                              __builtin_bit_cast(bf16x8, b[t2]), acc[t2], 0, 0, 0);
                        }
                    }
                }
            }
            if (st + 1 < stages) {
                // (more stages of this tile to come)
            } else if constexpr (!VEC) {
                store_tile<T, GELU>(p, acc, tile, tiles_per_img, m0, mt, ph, l32, half);
            } else if (m0 + 32 * mt < p.M) {  // wavefront-uniform
                // lane l of accumulator tile t holds output channel m0 + 32 mt + l % 32, pixels
                // 64 ph + 32 t + 8 q + 4 (l / 32) + (0 ... 3) in registers 4 q ... 4 q + 3
                typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
                const unsigned n = tile / tiles_per_img;
                const unsigned tpx = (tile - n * tiles_per_img) * kPwTile + 64 * ph;  // first pixel of the wavefront's 64
                const unsigned plane_bytes = (unsigned)p.P * 2u;
                const Rsrc rdst = __builtin_amdgcn_make_buffer_rsrc((void *)((T *)p.dst + (size_t)n * p.dst_img_stride), 0,
                                                                    (int)((unsigned)p.M * plane_bytes), kRawBuffer);
                const Rsrc rres = __builtin_amdgcn_make_buffer_rsrc(
                    (void *)((const T *)p.res + (size_t)n * p.res_img_stride), 0,
                    p.res != nullptr ? (int)((unsigned)p.M * plane_bytes) : 0, kRawBuffer);
                const unsigned co = (unsigned)(m0 + 32 * mt + l32);
                u32x2 rv[2][4];
#pragma unroll
                for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const unsigned px = tpx + 32 * t2 + 8 * q + 4 * half;  // P % 8 == 0: four pixels are inside or outside together
                        const unsigned off = px < (unsigned)p.P ? co * plane_bytes + px * 2u : kBeyond;
                        rv[t2][q] = __builtin_bit_cast(u32x2, __builtin_amdgcn_raw_buffer_load_b64(rres, (int)off, 0, kNt));
                    }
#pragma unroll
                for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        auto act = [](float a) { return GELU ? pw_gelu(a) : a; };
                        const float v0 = act(acc[t2][4 * q + 0]) + __uint_as_float(rv[t2][q].x << 16);
                        const float v1 = act(acc[t2][4 * q + 1]) + __uint_as_float(rv[t2][q].x & 0xffff0000u);
                        const float v2 = act(acc[t2][4 * q + 2]) + __uint_as_float(rv[t2][q].y << 16);
                        const float v3 = act(acc[t2][4 * q + 3]) + __uint_as_float(rv[t2][q].y & 0xffff0000u);
                        const u32x2 w = {pw_pack2_bf16(v0, v1), pw_pack2_bf16(v2, v3)};
                        *reinterpret_cast<u32x2 *>(s_o + l32 * kPwBfOPitch + 8 * ((4 * t2 + q) ^ (l32 & 7)) + 4 * half) = w;
                    }
                __builtin_amdgcn_wave_barrier();  // (the wavefront's LDS accesses are carried out in order)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int ch = 8 * i + (lane >> 3), piece = lane & 7;
                    const u32x4 v = *reinterpret_cast<const u32x4 *>(s_o + ch * kPwBfOPitch + 8 * (piece ^ (ch & 7)));
                    const unsigned px = tpx + 8 * piece;
                    const unsigned off = px < (unsigned)p.P ? (unsigned)(m0 + 32 * mt + ch) * plane_bytes + px * 2u : kBeyond;
                    __builtin_amdgcn_raw_buffer_store_b128(v, rdst, (int)off, 0, kNt);
                }
                __builtin_amdgcn_wave_barrier();
            }
            cur = next(cur);
            ahead = next(ahead);
            ++step;
        };
        while (cur.tile < n_tiles) {
            body(regs_a);
            if (cur.tile >= n_tiles) break;
            body(regs_b);
        }
    }
}

template <void (*KERNEL)(const PointwiseParams)>
hipError_t launch_one(const PointwiseParams &p, unsigned grid, size_t lds, hipStream_t s)
{
    static size_t granted = 48 * 1024;  // dynamic LDS a launch of this kernel may ask for without asking first
    if (lds > granted) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(KERNEL),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        granted = lds;
    }
    hipLaunchKernelGGL(KERNEL, dim3(grid), dim3(kPwThreads), lds, s, p);
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
    const size_t lds = bf16 ? kPwM * sizeof(float) + (2 * (size_t)kPwM * (Kr + 8) + 2 * (size_t)kPwKc * kPwBfBPitch +
                                                      4 * 32 * (size_t)kPwBfOPitch) * sizeof(uint16_t)
                            : ((size_t)Kr * kPwWPitch + kPwM + 2 * (size_t)kPwKc * kPwBPitch) * sizeof(float);
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
    if (p.gelu) {
        if (vec)
            return bf16 ? launch_one<pointwise_bf16_kernel<true, true>>(p, (unsigned)grid, lds, s)
                        : launch_one<pointwise_kernel<float, true, true>>(p, (unsigned)grid, lds, s);
        return bf16 ? launch_one<pointwise_bf16_kernel<false, true>>(p, (unsigned)grid, lds, s)
                    : launch_one<pointwise_kernel<float, false, true>>(p, (unsigned)grid, lds, s);
    }
    if (vec)
        return bf16 ? launch_one<pointwise_bf16_kernel<true, false>>(p, (unsigned)grid, lds, s)
                    : launch_one<pointwise_kernel<float, true, false>>(p, (unsigned)grid, lds, s);
    return bf16 ? launch_one<pointwise_bf16_kernel<false, false>>(p, (unsigned)grid, lds, s)
                : launch_one<pointwise_kernel<float, false, false>>(p, (unsigned)grid, lds, s);
}

}  // namespace esc

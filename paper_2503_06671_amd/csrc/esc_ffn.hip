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

// two fp32 values rounded to nearest even and packed, a in the low half: the hardware's
// packed conversion (v_cvt_pk_bf16_f32), one instruction where the shifts and adds above are a dozen
typedef float fb_f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 fb_bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t fb_pack2_bf16(float a, float b)
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(fb_f32x2{a, b}, fb_bf16x2));
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
                    w = u32x4{fb_pack2_bf16(o[0], o[1]), fb_pack2_bf16(o[2], o[3]), fb_pack2_bf16(o[4], o[5]),
                              fb_pack2_bf16(o[6], o[7])};
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


// ---- the whole network in one kernel (fp32 storage, C <= 64, Ch <= 128) ------------------
//
// A block streams down a strip of the image 32 columns wide (30 output columns and one
// halo column each side) over a band of rows.  Per input row y:
//   1. the row's C x 32 values are in LDS (fetched a row ahead), each as three bf16 terms
//      (v = t0 + t1 + t2 but for 2^-24 of it), pixel-major;
//   2. wavefront w forms U[32 w .. 32 w + 31][32 columns] = gelu(W1 . x + b1) with
//      v_mfma_f32_32x32x16_bf16 on the terms - its 32 x 64 tile of W1, three bf16 terms per
//      weight, lives in registers in the A operand's layout; six of the nine products of
//      terms are accumulated in fp32, what is left out lies below 2^-24 of a product: fp32
//      accuracy (3.8e-7 against the oracle at 180 x 320) from instructions a sixteenth as long
//      as the fp32 ones, which moreover do not hold up the vector units - and writes it,
//      zeroed outside the image (the branch pads U with zeros), into row y's slot of a
//      three-row ring in LDS;
//   3. the same wavefront applies the depth-wise branch to its own 32 hidden channels for
//      output row y - 1 (lane = one channel and sixteen columns; rows y - 2, y - 1, y from the
//      ring) and writes V over the ring's oldest row: the first layer, the GELU, the ring
//      and the branch never leave the wavefront, so no block barrier is needed up to here;
//   4. after a barrier, wavefront (mt, kh) multiplies W2's rows 32 mt .. + 31 with the 64
//      hidden channels 64 kh .. + 63 of V (v_mfma_f32_32x32x2_f32, its 32 x 64 tile of W2 in
//      registers: V as three pixel-major bf16 terms would not fit beside the ring with two
//      blocks per compute unit); the kh = 1 wavefronts hand their partial sums over through
//      LDS, the kh = 0 ones add them and b2 and store 30 columns of output row y - 1 - while
//      the kh = 1 ones already start on the next row.
// Two barriers per row, 73 KB of LDS (two blocks per compute unit), weights read once per
// block.  The band's first two input rows are recomputed by the band above
// (rows_per_band + 2 first-layer rows for rows_per_band output rows), the strips' halo
// columns by their neighbours (32 for 30).  Measured: fp32 matrix instructions' time and
// the vector instructions' time add up in this kernel - neither issued among the other
// wavefront's nor among the same wavefront's vector instructions do fp32 matrix
// instructions run beside them - so the phases are simply written one after the other,
// and the first layer moved to the bf16 instructions (46.8 -> 41.0 us at 180 x 320).

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u32x4s __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8s __attribute__((ext_vector_type(8)));

constexpr int kFsThreads = 256;
constexpr int kFsC = 64;        // input (and output) channels the tiles hold
constexpr int kFsCh = 128;      // hidden channels the tiles hold
constexpr int kFsNp = 32;       // columns of a strip, halo included
constexpr int kFsOut = 30;      // output columns of a strip
constexpr int kFsPitch = 33;    // floats between two channel rows of the ring (odd: lanes on different channels, same column, hit different banks)
constexpr int kFsXPitch = kFsC + 8;                       // bf16 elements between two columns of the input row tile (144 bytes)
constexpr int kFsXTerm = kFsNp * kFsXPitch;               // bf16 elements of one term's tile
constexpr int kFsXFloats = (3 * kFsXTerm * 2 + 3) / 4;    // the input row as three bf16 terms, pixel-major (one buffer)
static_assert((3 * kFsXTerm * 2) % 16 == 0, "the ring starts on a 16-byte boundary");
constexpr int kFsRingFloats = 3 * kFsCh * kFsPitch;
constexpr int kFsRedFloats = 2 * 16 * 64;
constexpr int kFsBiasFloats = kFsCh + kFsC;
constexpr size_t kFsLdsBytes = (size_t)(kFsXFloats + kFsRingFloats + kFsRedFloats + kFsBiasFloats) * sizeof(float);

static_assert(kFsCh * (kFsC + 1) + kFsC * (kFsCh + 1) <= kFsXFloats + kFsRingFloats + kFsRedFloats,
              "the weights pass through the row tile's, the ring's and the partial sums' space on their way into registers");

extern __shared__ __align__(16) float fs_lds[];

__global__ __launch_bounds__(kFsThreads, 2) void ffn_stream_kernel(const FfnStreamParams p)
{
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int mt = wave & 1, kh = wave >> 1;
    const int C = p.C, Ch = p.Ch, H = p.H, W = p.W;

    uint16_t *sX = reinterpret_cast<uint16_t *>(fs_lds);   // [3 terms][kFsNp][kFsXPitch] bf16
    float *ring = fs_lds + kFsXFloats;      // [3][kFsCh][kFsPitch]
    float *red = ring + kFsRingFloats;      // [2 mt][16][64]
    float *sB1 = red + kFsRedFloats;        // [kFsCh] first layer's biases, zeros beyond Ch
    float *sB2 = sB1 + kFsCh;               // [kFsC] second layer's

    // which strip, band and image.  Blocks are dealt to the eight dies (XCDs) in turn, each die
    // with an L2 of its own: block b works on piece (b % 8) * (grid / 8) + b / 8 of the image, so
    // that neighbouring strips and bands - which share cache lines (a strip's 128-byte row
    // segments start one column left of a 30-column boundary) and halo rows - meet in one L2
    const unsigned bq = gridDim.x / 8u, br = gridDim.x % 8u, xcd = blockIdx.x % 8u;
    const unsigned piece = xcd * bq + (xcd < br ? xcd : br) + blockIdx.x / 8u;
    const unsigned per_img = (unsigned)p.strips * (unsigned)p.bands;
    const unsigned n = piece / per_img;
    const unsigned rem = piece - n * per_img;
    const int band = (int)(rem / (unsigned)p.strips), strip = (int)(rem - (unsigned)band * (unsigned)p.strips);
    const int x0 = strip * kFsOut - 1;                    // image column of the strip's column 0
    const int y0 = band * p.rows_per_band;                // first output row
    const int rows_out = min(p.rows_per_band, H - y0);    // >= 1
    const size_t plane = (size_t)H * W;
    const float *xin = (const float *)p.x + (size_t)n * C * plane;
    const unsigned plane_bytes = (unsigned)plane * 4u;
    const __amdgpu_buffer_rsrc_t rout = __builtin_amdgcn_make_buffer_rsrc((void *)((float *)p.out + (size_t)n * C * plane), 0,
                                                                          (int)((unsigned)C * plane_bytes), 0x00020000);

    // ---- this thread's share of an input row: column tid % 32 of channels tid / 32 + 8 i ----
    const int xpx = tid & 31, xc0 = tid >> 5;
    const int gx_in = x0 + xpx;
    const bool col_in = gx_in >= 0 && gx_in < W;
    // (the loads' results are not touched until they are put into LDS a row later: a value
    // used right behind its load makes the compiler wait for the load there)
    auto fetch_row = [&](int gy, float (&v)[8]) {
        const bool row_in = gy >= 0 && gy < H;
        const size_t off = (size_t)(row_in ? gy : 0) * W + (size_t)(col_in ? gx_in : 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int c = xc0 + 8 * i;
            v[i] = xin[(size_t)(c < C ? c : 0) * plane + off];
        }
    };
    // a row into LDS as three bf16 terms per value (v = t0 + t1 + t2 but for 2^-24 of it: each term
    // the nearest bf16 to what the terms before it left), pixel-major: the first layer's B operands
    auto put_row = [&](const float (&v)[8], int gy) {
        const bool in = col_in && gy >= 0 && gy < H;
        uint16_t *d = sX + xpx * kFsXPitch + xc0;
#pragma unroll
        for (int i = 0; i < 8; i += 2) {
            const float v0 = (in && xc0 + 8 * i < C) ? v[i] : 0.f, v1 = (in && xc0 + 8 * (i + 1) < C) ? v[i + 1] : 0.f;
            const uint32_t t0 = fb_pack2_bf16(v0, v1);
            const float r0 = v0 - __uint_as_float(t0 << 16), r1 = v1 - __uint_as_float(t0 & 0xffff0000u);
            const uint32_t t1 = fb_pack2_bf16(r0, r1);
            const uint32_t t2 = fb_pack2_bf16(r0 - __uint_as_float(t1 << 16), r1 - __uint_as_float(t1 & 0xffff0000u));
            d[8 * i] = (uint16_t)t0, d[8 * (i + 1)] = (uint16_t)(t0 >> 16);
            d[kFsXTerm + 8 * i] = (uint16_t)t1, d[kFsXTerm + 8 * (i + 1)] = (uint16_t)(t1 >> 16);
            d[2 * kFsXTerm + 8 * i] = (uint16_t)t2, d[2 * kFsXTerm + 8 * (i + 1)] = (uint16_t)(t2 >> 16);
        }
    };

    float xr[8];
    fetch_row(y0 - 1, xr);  // the band's first input row travels while the weights are staged

    // ---- weights into registers, in the matrix instructions' A layout.  They pass through
    // LDS (the row buffers' and the ring's space, rows of an odd pitch), fetched by the block with coalesced loads:
    // fetched by every lane for itself - thirty-two rows per load instruction - the blocks
    // moved half a gigabyte through the L2 for 64 KB of weights ----
    // first layer (bf16 instructions on exact terms): lane holds W1[32 w + l32][16 c + 8 half ... + 7] of
    // chunk c as three bf16 terms; second layer (fp32 instructions): W2[32 mt + l32][64 kh + 2 kp + half]
    u32x4s a1t[3][4];
    float a2[32];
    {
        constexpr int kP1 = kFsC + 1, kP2 = kFsCh + 1;
        float *s1 = fs_lds, *s2 = fs_lds + kFsCh * kP1;  // both matrices at once, over the row buffers and the ring
        for (int i0 = tid; i0 < kFsCh * kFsC; i0 += 8 * kFsThreads) {
            float v[8], w[8];
            bool in1[8], in2[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {  // sixteen loads out together, their uses behind them
                const int i = i0 + u * kFsThreads;
                const int r1 = i / kFsC, c1 = i - r1 * kFsC, r2 = i / kFsCh, c2 = i - r2 * kFsCh;
                in1[u] = r1 < Ch && c1 < C;
                in2[u] = r2 < C && c2 < Ch;
                v[u] = p.w1[in1[u] ? (size_t)r1 * C + c1 : 0];
                w[u] = p.w2[in2[u] ? (size_t)r2 * Ch + c2 : 0];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + u * kFsThreads;
                const int r1 = i / kFsC, c1 = i - r1 * kFsC, r2 = i / kFsCh, c2 = i - r2 * kFsCh;
                s1[r1 * kP1 + c1] = in1[u] ? v[u] : 0.f;
                s2[r2 * kP2 + c2] = in2[u] ? w[u] : 0.f;
            }
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            unsigned t[3][4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float w0 = s1[(32 * wave + l32) * kP1 + 16 * c + 8 * half + 2 * e];
                const float w1 = s1[(32 * wave + l32) * kP1 + 16 * c + 8 * half + 2 * e + 1];
                t[0][e] = fb_pack2_bf16(w0, w1);
                const float r0 = w0 - __uint_as_float(t[0][e] << 16), r1 = w1 - __uint_as_float(t[0][e] & 0xffff0000u);
                t[1][e] = fb_pack2_bf16(r0, r1);
                t[2][e] = fb_pack2_bf16(r0 - __uint_as_float(t[1][e] << 16), r1 - __uint_as_float(t[1][e] & 0xffff0000u));
            }
#pragma unroll
            for (int q = 0; q < 3; ++q) a1t[q][c] = u32x4s{t[q][0], t[q][1], t[q][2], t[q][3]};
        }
#pragma unroll
        for (int kp = 0; kp < 32; ++kp) a2[kp] = s2[(32 * mt + l32) * kP2 + 64 * kh + 2 * kp + half];
        __syncthreads();  // everyone has its weights: the space is the row buffers' and the ring's from here on
    }
    // biases into LDS (the first barrier below covers them)
    if (tid < kFsCh) sB1[tid] = (p.b1 != nullptr && tid < Ch) ? p.b1[tid] : 0.f;
    if (tid < kFsC) sB2[tid] = (p.b2 != nullptr && tid < C) ? p.b2[tid] : 0.f;
    // the branch: lane = hidden channel 32 w + l32, columns 16 half .. 16 half + 15 of the strip
    const int chb = 32 * wave + l32;
    float kd[9], bkd;
    {
        const bool in = chb < Ch;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const float v = p.k[in ? (size_t)chb * 9 + t : 0];
            kd[t] = in ? v : 0.f;
        }
        const float vb = p.bk != nullptr ? p.bk[in ? chb : 0] : 0.f;
        bkd = (in && p.bk != nullptr) ? vb : 0.f;
    }

    put_row(xr, y0 - 1);
    fetch_row(y0, xr);
    __syncthreads();

    const bool ucol_in = (x0 + l32) >= 0 && (x0 + l32) < W;   // the column a lane's accumulators hold
    const int steps = rows_out + 2;
    for (int r = 0; r < steps; ++r) {
        const int gy = y0 - 1 + r;   // this step's input row
        // ---- first layer on row gy: U tile = W1 tile . x row ----
        {
            f32x16 acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = 0.f;
            // the biases of the rows this lane's accumulators hold, asked for in front of the
            // products (read one by one where they are used, each read's latency was waited for)
            const float *b1p = sB1 + 32 * wave + 4 * half;
            float b1v[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) b1v[i] = b1p[8 * (i >> 2) + (i & 3)];
            // v_mfma_f32_32x32x16_bf16 on the terms: of the nine products of a weight's and a value's terms
            // the six whose orders add up to at most two (the rest lies below 2^-24 of a product)
            const uint16_t *bx = sX + l32 * kFsXPitch + 8 * half;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                u32x4s x3[3];
#pragma unroll
                for (int q = 0; q < 3; ++q) x3[q] = *reinterpret_cast<const u32x4s *>(bx + q * kFsXTerm + 16 * c);
#pragma unroll
                for (int qw = 2; qw >= 0; --qw)
#pragma unroll
                    for (int qx = 2 - qw; qx >= 0; --qx)
                        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8s, a1t[qw][c]),
                                                                      __builtin_bit_cast(bf16x8s, x3[qx]), acc, 0, 0, 0);
            }
            const bool live = ucol_in && gy >= 0 && gy < H;
            float *ur = ring + (r % 3) * (kFsCh * kFsPitch) + (32 * wave + 4 * half) * kFsPitch + l32;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int m = 8 * (i >> 2) + (i & 3);   // (+ 4 half: in ur and b1p)
                const float u = fb_gelu(acc[i] + b1v[i]);
                ur[m * kFsPitch] = live ? u : 0.f;
            }
        }
        __builtin_amdgcn_wave_barrier();  // (a wavefront's LDS accesses are carried out in order)
        // ---- the branch on output row gy - 1, this wavefront's 32 hidden channels ----
        const int vslot = (r + 1) % 3;    // the ring's oldest row, (r - 2) % 3: V goes there
        if (r >= 2) {
            float a[3][18];
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                const float *row = ring + ((r + 1 + i) % 3) * (kFsCh * kFsPitch) + chb * kFsPitch;
#pragma unroll
                for (int j = 0; j < 18; ++j) {
                    const int px = 16 * half - 1 + j;   // -1 and 32 lie outside the strip: only halo columns need them
                    const float v = row[px < 0 ? 0 : (px > 31 ? 31 : px)];
                    a[i][j] = (px >= 0 && px <= 31) ? v : 0.f;
                }
            }
            float vv[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                float s = bkd;
                s = fmaf(kd[0], a[0][j], s), s = fmaf(kd[1], a[0][j + 1], s), s = fmaf(kd[2], a[0][j + 2], s);
                s = fmaf(kd[3], a[1][j], s), s = fmaf(kd[4], a[1][j + 1], s), s = fmaf(kd[5], a[1][j + 2], s);
                s = fmaf(kd[6], a[2][j], s), s = fmaf(kd[7], a[2][j + 1], s), s = fmaf(kd[8], a[2][j + 2], s);
                vv[j] = a[1][j + 1] + fb_gelu(s);
            }
            __builtin_amdgcn_wave_barrier();  // every lane has read the oldest row before any lane overwrites it
            float *vr = ring + vslot * (kFsCh * kFsPitch) + chb * kFsPitch + 16 * half;
#pragma unroll
            for (int j = 0; j < 16; ++j) vr[j] = vv[j];
        }
        __syncthreads();  // V of all hidden channels is in LDS; everyone has multiplied this step's input row
        // the next row into the (one) row tile, the row after it asked for
        if (r + 1 < steps) {
            put_row(xr, gy + 1);
            if (r + 2 < steps) fetch_row(gy + 2, xr);
        }
        // ---- second layer: W2 tile (32 output channels x 64 hidden channels) . V ----
        f32x16 acc2;
        if (r >= 2) {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc2[i] = 0.f;
            const float *bv = ring + vslot * (kFsCh * kFsPitch) + (64 * kh + half) * kFsPitch + l32;
#pragma unroll
            for (int kp = 0; kp < 32; ++kp)
                acc2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a2[kp], bv[2 * kp * kFsPitch], acc2, 0, 0, 0);
            if (kh == 1) {
#pragma unroll
                for (int i = 0; i < 16; ++i) red[(mt * 16 + i) * 64 + lane] = acc2[i];
            }
        }
        __syncthreads();  // the partial sums and the next input row are in LDS; nobody reads V any more
        if (r >= 2 && kh == 0) {
            const int gyo = gy - 1, gxo = x0 + l32;
            const bool st_ok = l32 >= 1 && l32 <= kFsOut && gxo < W;   // (gyo < H by the loop's bound)
            float rv[16], bv[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                rv[i] = red[(mt * 16 + i) * 64 + lane];
                bv[i] = sB2[32 * mt + 8 * (i >> 2) + 4 * half + (i & 3)];
            }
            // buffer stores on a resource that is the image's output: what is not to be
            // written gets an offset beyond it and is dropped - no branches
            // (the channel's plane offset as the lane's part plus a multiple of the plane's bytes that is
            // the same for all lanes: one multiplication per lane instead of sixteen)
            const int co0 = 32 * mt + 4 * half;
            const unsigned lane_off = (unsigned)co0 * plane_bytes + (unsigned)(gyo * W + gxo) * 4u;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int dc = 8 * (i >> 2) + (i & 3);
                const float v = acc2[i] + rv[i] + bv[i];
                const unsigned off = (st_ok && co0 + dc < C) ? lane_off + (unsigned)dc * plane_bytes : 0x80000000u;
                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), rout, (int)off, 0, 2 /* non-temporal */);
            }
        }
    }
}

// ---- the same for bf16 storage, on the bf16 matrix instructions --------------------------
//
// v_mfma_f32_32x32x16_bf16 on the stored values, every fp32 weight as two bf16 terms
// (w = hi + lo to 16 mantissa bits; products exact, fp32 accumulation): a sixteenth of the
// fp32 instructions' time, and beside the vector units instead of in their way.  What
// changes against the fp32 kernel is the layout of the matrix operands: an operand wants
// eight consecutive channels of one pixel per lane, so the input row and V sit in LDS
// pixel-major ([column][channel] bf16, 16-byte reads; pitches of 4 words mod 32, which
// spreads a half-wavefront's sixteen-byte reads evenly over the banks), each weight tile is
// 2 terms x 4 chunks of sixteen channels x 4 registers, and V has a buffer of its own (it
// is bf16, the ring fp32).  U stays fp32 in the ring - only V is rounded to bf16 on the way
// to the second layer, as a stored V would be - and out is rounded once at its store.

constexpr int kFbXPitch = kFsC + 8;                  // bf16 elements between two columns of an input row tile (144 bytes)
constexpr int kFbVPitch = kFsCh + 8;                 // ... of V's tile (272 bytes)
constexpr int kFbXElems = 2 * kFsNp * kFbXPitch;     // two row buffers
constexpr int kFbVElems = kFsNp * kFbVPitch;
constexpr size_t kFbLdsBytes = (size_t)(kFbXElems + kFbVElems) * 2 +
                               (size_t)(kFsRingFloats + kFsRedFloats + kFsBiasFloats) * sizeof(float);
static_assert((kFbXElems * 2) % 16 == 0 && (kFbVElems * 2) % 16 == 0, "the fp32 parts start on 16-byte boundaries");
static_assert((size_t)(kFsCh * (kFsC + 1) + kFsC * (kFsCh + 1)) * 4 <= (size_t)(kFbXElems + kFbVElems) * 2 + (size_t)kFsRingFloats * 4,
              "the weights pass through the tiles' and the ring's space on their way into registers");

// eight fp32 weights as the two bf16 terms of an A operand: hi = bf16(w), lo = bf16(w - hi)
__device__ __forceinline__ void fb_split8(const float *w, u32x4s &hi, u32x4s &lo)
{
    unsigned h[4], l[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        h[e] = fb_pack2_bf16(w[2 * e], w[2 * e + 1]);
        l[e] = fb_pack2_bf16(w[2 * e] - __uint_as_float(h[e] << 16), w[2 * e + 1] - __uint_as_float(h[e] & 0xffff0000u));
    }
    hi = u32x4s{h[0], h[1], h[2], h[3]};
    lo = u32x4s{l[0], l[1], l[2], l[3]};
}

__global__ __launch_bounds__(kFsThreads, 2) void ffn_stream_bf16_kernel(const FfnStreamParams p)
{
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int mt = wave & 1, kh = wave >> 1;
    const int C = p.C, Ch = p.Ch, H = p.H, W = p.W;

    uint16_t *sX = reinterpret_cast<uint16_t *>(fs_lds);   // [2][kFsNp][kFbXPitch] bf16
    uint16_t *sV = sX + kFbXElems;                         // [kFsNp][kFbVPitch] bf16
    float *ring = reinterpret_cast<float *>(sV + kFbVElems);  // [3][kFsCh][kFsPitch]
    float *red = ring + kFsRingFloats;                     // [2 mt][16][64]
    float *sB1 = red + kFsRedFloats;
    float *sB2 = sB1 + kFsCh;

    // which strip, band and image (pieces dealt so that neighbours meet in one die's L2, as above)
    const unsigned bq = gridDim.x / 8u, br = gridDim.x % 8u, xcd = blockIdx.x % 8u;
    const unsigned piece = xcd * bq + (xcd < br ? xcd : br) + blockIdx.x / 8u;
    const unsigned per_img = (unsigned)p.strips * (unsigned)p.bands;
    const unsigned n = piece / per_img;
    const unsigned rem = piece - n * per_img;
    const int band = (int)(rem / (unsigned)p.strips), strip = (int)(rem - (unsigned)band * (unsigned)p.strips);
    const int x0 = strip * kFsOut - 1;
    const int y0 = band * p.rows_per_band;
    const int rows_out = min(p.rows_per_band, H - y0);
    const size_t plane = (size_t)H * W;
    const uint16_t *xin = (const uint16_t *)p.x + (size_t)n * C * plane;
    const unsigned plane_bytes = (unsigned)plane * 2u;
    const __amdgpu_buffer_rsrc_t rout = __builtin_amdgcn_make_buffer_rsrc((void *)((uint16_t *)p.out + (size_t)n * C * plane), 0,
                                                                          (int)((unsigned)C * plane_bytes), 0x00020000);

    // ---- this thread's share of an input row: column tid % 32 of channels tid / 32 + 8 i ----
    const int xpx = tid & 31, xc0 = tid >> 5;
    const int gx_in = x0 + xpx;
    const bool col_in = gx_in >= 0 && gx_in < W;
    auto fetch_row = [&](int gy, uint16_t (&v)[8]) {
        const bool row_in = gy >= 0 && gy < H;
        const size_t off = (size_t)(row_in ? gy : 0) * W + (size_t)(col_in ? gx_in : 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int c = xc0 + 8 * i;
            v[i] = xin[(size_t)(c < C ? c : 0) * plane + off];
        }
    };
    auto put_row = [&](const uint16_t (&v)[8], int gy, int buf) {
        const bool in = col_in && gy >= 0 && gy < H;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            sX[buf * (kFsNp * kFbXPitch) + xpx * kFbXPitch + xc0 + 8 * i] = (in && xc0 + 8 * i < C) ? v[i] : (uint16_t)0;
    };

    uint16_t xr[8];
    fetch_row(y0 - 1, xr);  // the band's first input row travels while the weights are staged

    // ---- weights: fp32 through LDS as in the fp32 kernel, then split into their two bf16
    // terms in the A operand's layout: lane holds W[row][16 c + 8 half ... + 7] of chunk c ----
    u32x4s a1h[4], a1l[4], a2h[4], a2l[4];
    {
        constexpr int kP1 = kFsC + 1, kP2 = kFsCh + 1;
        float *s1 = fs_lds, *s2 = fs_lds + kFsCh * kP1;
        for (int i0 = tid; i0 < kFsCh * kFsC; i0 += 8 * kFsThreads) {
            float v[8], w[8];
            bool in1[8], in2[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + u * kFsThreads;
                const int r1 = i / kFsC, c1 = i - r1 * kFsC, r2 = i / kFsCh, c2 = i - r2 * kFsCh;
                in1[u] = r1 < Ch && c1 < C;
                in2[u] = r2 < C && c2 < Ch;
                v[u] = p.w1[in1[u] ? (size_t)r1 * C + c1 : 0];
                w[u] = p.w2[in2[u] ? (size_t)r2 * Ch + c2 : 0];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + u * kFsThreads;
                const int r1 = i / kFsC, c1 = i - r1 * kFsC, r2 = i / kFsCh, c2 = i - r2 * kFsCh;
                s1[r1 * kP1 + c1] = in1[u] ? v[u] : 0.f;
                s2[r2 * kP2 + c2] = in2[u] ? w[u] : 0.f;
            }
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float w8[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) w8[e] = s1[(32 * wave + l32) * kP1 + 16 * c + 8 * half + e];
            fb_split8(w8, a1h[c], a1l[c]);
#pragma unroll
            for (int e = 0; e < 8; ++e) w8[e] = s2[(32 * mt + l32) * kP2 + 64 * kh + 16 * c + 8 * half + e];
            fb_split8(w8, a2h[c], a2l[c]);
        }
        __syncthreads();  // everyone has its weights: the space is the tiles' and the ring's from here on
    }
    if (tid < kFsCh) sB1[tid] = (p.b1 != nullptr && tid < Ch) ? p.b1[tid] : 0.f;
    if (tid < kFsC) sB2[tid] = (p.b2 != nullptr && tid < C) ? p.b2[tid] : 0.f;
    const int chb = 32 * wave + l32;
    float kd[9], bkd;
    {
        const bool in = chb < Ch;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const float v = p.k[in ? (size_t)chb * 9 + t : 0];
            kd[t] = in ? v : 0.f;
        }
        const float vb = p.bk != nullptr ? p.bk[in ? chb : 0] : 0.f;
        bkd = (in && p.bk != nullptr) ? vb : 0.f;
    }

    put_row(xr, y0 - 1, 0);
    fetch_row(y0, xr);
    __syncthreads();

    const bool ucol_in = (x0 + l32) >= 0 && (x0 + l32) < W;
    const int steps = rows_out + 2;
    for (int r = 0; r < steps; ++r) {
        const int gy = y0 - 1 + r;
        if (r + 1 < steps) {
            put_row(xr, gy + 1, (r + 1) & 1);
            if (r + 2 < steps) fetch_row(gy + 2, xr);
        }
        // ---- first layer on row gy ----
        {
            f32x16 acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = 0.f;
            const uint16_t *bx = sX + (r & 1) * (kFsNp * kFbXPitch) + l32 * kFbXPitch + 8 * half;
            const float *b1p = sB1 + 32 * wave + 4 * half;
            float b1v[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) b1v[i] = b1p[8 * (i >> 2) + (i & 3)];
            u32x4s bq[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) bq[c] = *reinterpret_cast<const u32x4s *>(bx + 16 * c);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8s, a1h[c]), __builtin_bit_cast(bf16x8s, bq[c]), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8s, a1l[c]), __builtin_bit_cast(bf16x8s, bq[c]), acc, 0, 0, 0);
            }
            const bool live = ucol_in && gy >= 0 && gy < H;
            float *ur = ring + (r % 3) * (kFsCh * kFsPitch) + (32 * wave + 4 * half) * kFsPitch + l32;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int m = 8 * (i >> 2) + (i & 3);
                const float u = fb_gelu(acc[i] + b1v[i]);
                ur[m * kFsPitch] = live ? u : 0.f;
            }
        }
        __builtin_amdgcn_wave_barrier();  // (a wavefront's LDS accesses are carried out in order)
        // ---- the branch on output row gy - 1; V, rounded to bf16, into its pixel-major tile ----
        if (r >= 2) {
            float a[3][18];
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                const float *row = ring + ((r + 1 + i) % 3) * (kFsCh * kFsPitch) + chb * kFsPitch;
#pragma unroll
                for (int j = 0; j < 18; ++j) {
                    const int px = 16 * half - 1 + j;
                    const float v = row[px < 0 ? 0 : (px > 31 ? 31 : px)];
                    a[i][j] = (px >= 0 && px <= 31) ? v : 0.f;
                }
            }
            uint16_t *vr = sV + (16 * half) * kFbVPitch + chb;
            float vv[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                float s = bkd;
                s = fmaf(kd[0], a[0][j], s), s = fmaf(kd[1], a[0][j + 1], s), s = fmaf(kd[2], a[0][j + 2], s);
                s = fmaf(kd[3], a[1][j], s), s = fmaf(kd[4], a[1][j + 1], s), s = fmaf(kd[5], a[1][j + 2], s);
                s = fmaf(kd[6], a[2][j], s), s = fmaf(kd[7], a[2][j + 1], s), s = fmaf(kd[8], a[2][j + 2], s);
                vv[j] = a[1][j + 1] + fb_gelu(s);
            }
#pragma unroll
            for (int j = 0; j < 16; j += 2) {
                const uint32_t pk = fb_pack2_bf16(vv[j], vv[j + 1]);
                vr[j * kFbVPitch] = (uint16_t)pk;
                vr[(j + 1) * kFbVPitch] = (uint16_t)(pk >> 16);
            }
        }
        __syncthreads();  // V of all hidden channels (and the next input row) is in LDS
        // ---- second layer ----
        f32x16 acc2;
        if (r >= 2) {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc2[i] = 0.f;
            const uint16_t *bv = sV + l32 * kFbVPitch + 64 * kh + 8 * half;
            u32x4s vq[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) vq[c] = *reinterpret_cast<const u32x4s *>(bv + 16 * c);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                acc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8s, a2h[c]), __builtin_bit_cast(bf16x8s, vq[c]), acc2, 0, 0, 0);
                acc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8s, a2l[c]), __builtin_bit_cast(bf16x8s, vq[c]), acc2, 0, 0, 0);
            }
            if (kh == 1) {
#pragma unroll
                for (int i = 0; i < 16; ++i) red[(mt * 16 + i) * 64 + lane] = acc2[i];
            }
        }
        __syncthreads();  // the partial sums are in LDS; nobody reads V any more
        if (r >= 2 && kh == 0) {
            const int gyo = gy - 1, gxo = x0 + l32;
            const bool st_ok = l32 >= 1 && l32 <= kFsOut && gxo < W;
            float rv[16], bv2[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                rv[i] = red[(mt * 16 + i) * 64 + lane];
                bv2[i] = sB2[32 * mt + 8 * (i >> 2) + 4 * half + (i & 3)];
            }
            const int co0 = 32 * mt + 4 * half;
            const unsigned lane_off = (unsigned)co0 * plane_bytes + (unsigned)(gyo * W + gxo) * 2u;
#pragma unroll
            for (int i = 0; i < 16; i += 2) {
                const uint32_t pk = fb_pack2_bf16(acc2[i] + rv[i] + bv2[i], acc2[i + 1] + rv[i + 1] + bv2[i + 1]);
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const int dc = 8 * ((i + e) >> 2) + ((i + e) & 3);
                    const unsigned off = (st_ok && co0 + dc < C) ? lane_off + (unsigned)dc * plane_bytes : 0x80000000u;
                    __builtin_amdgcn_raw_buffer_store_b16((unsigned short)(e == 0 ? pk : pk >> 16), rout, (int)off, 0, 2 /* non-temporal */);
                }
            }
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

__attribute__((visibility("hidden"))) hipError_t launch_ffn_stream(const FfnStreamParams &p, hipStream_t s)
{
    if (p.N < 1 || p.C < 1 || p.H < 1 || p.W < 1 || p.Ch < 1) return hipSuccess;
    if (p.C > kFsC || p.Ch > kFsCh) return hipErrorNotSupported;
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return hipErrorInvalidDevice;
        cus = n > 0 ? n : 1;
    }
    static bool lds_granted = false;
    if (!lds_granted) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(ffn_stream_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFsLdsBytes);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(ffn_stream_bf16_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFbLdsBytes);
        if (e != hipSuccess) return e;
        lds_granted = true;
    }
    FfnStreamParams q = p;
    q.strips = (p.W + kFsOut - 1) / kFsOut;
    // a block lasts as long whatever the image's size (its weights' way into registers, then six
    // rows one after the other): with too few blocks to fill the chip the three launches are faster
    if ((long)p.N * q.strips * ((p.H + 3) / 4) < 3L * cus / 2) return hipErrorNotSupported;
    // ... and a last strip that is mostly empty costs as much as a full one: widths that fill less than
    // four fifths of their strips keep the three launches too (64 columns are 30 + 30 + 4)
    if (5L * p.W < 4L * q.strips * kFsOut) return hipErrorNotSupported;
    // the band height that needs the fewest row steps one after the other: a block takes its rows + 2
    // steps and about a step and a half to get its weights; the blocks run in rounds of two per compute unit
    q.rows_per_band = 4;
    double best = 0.0;
    for (int rb = 4; rb <= 32; rb *= 2) {
        const long blocks = (long)p.N * q.strips * ((p.H + rb - 1) / rb);
        const long rounds = (blocks + 2L * cus - 1) / (2L * cus);
        const double cost = (double)rounds * (rb + 3.5);
        if (rb == 4 || cost < best) {
            best = cost;
            q.rows_per_band = rb;
        }
    }
    q.bands = (p.H + q.rows_per_band - 1) / q.rows_per_band;
    const long grid = (long)p.N * q.strips * q.bands;
    if (grid >= (1L << 31)) return hipErrorNotSupported;
    if (p.bf16)
        hipLaunchKernelGGL(ffn_stream_bf16_kernel, dim3((unsigned)grid), dim3(kFsThreads), kFbLdsBytes, s, q);
    else
        hipLaunchKernelGGL(ffn_stream_kernel, dim3((unsigned)grid), dim3(kFsThreads), kFsLdsBytes, s, q);
    return hipGetLastError();
}

}  // namespace esc

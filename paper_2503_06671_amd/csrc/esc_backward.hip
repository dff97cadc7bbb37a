// Backward pass of the ConvAttn module (depth-wise form; Eq. 4 lines 1-4 of the ESC paper
// without Conv_fuse) for gfx950 (MI355X).  The paper trains its shared LK end to end
// (Sec. 3) but prints no gradient formulae; these are the derivatives of the definition:
//
//   S[n,c,i,j]  = sum_{y,x} go[n,c,y,x] xz[n,c,y+i-p,x+j-p]      correlation of grad_out with x
//   dLK[c]      = sum_n S[n,c]           dDK[n,c] = centre 3 x 3 of S[n,c]
//   estimator   : dd = dDK;  db_up = sum_n dd;  dw_up = sum_n dd (x) t;  dt = w_up^T dd;
//                 du = dt * gelu'(u);  db_down = sum_n du;  dw_down = sum_n du (x) g;  dg = w_down^T du
//   dx[n,c]     = go[n,c] (*) flip(LK[c] + ZP(DK[n,c])) + dg[n,c] / (H W)     (c < C_a; dx = go elsewhere)
//
// The input gradient's convolution is the forward kernel itself, run on grad_out with the
// flipped kernels (esc_api.hip); this file holds what is new: the correlation S - windows up
// to 15 x 15 as Toeplitz products on the matrix cores (corr_mfma_kernel), larger ones with
// the forward's vector tap loop turned round (corr_kernel: 2 Ks^2 flops per pixel into Ks^2
// sums) - and the small estimator kernels; the GAP term of dx is a constant per plane that the
// input gradient's launch adds at its stores.  Every sum has a fixed order
// (per-tile partial sums in the workspace, then one thread per result), so results do not
// depend on scheduling.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "esc_backward.hpp"

namespace esc {
namespace {

constexpr int kBwThreads = 256;

struct bf16b {
    uint16_t bits;
};
__device__ __forceinline__ float bw_load(const float *p) { return *p; }
__device__ __forceinline__ float bw_load(const bf16b *p) { return __uint_as_float((uint32_t)p->bits << 16); }
__device__ __forceinline__ uint16_t bw_f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// running sum along each row of 16 lanes (data-parallel moves inside the vector unit):
// lane 15 of a row ends with the row's total, in a fixed order
__device__ __forceinline__ float row16_sum(float v)
{
    auto dpp = [](float x, auto ctrl) {
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value,
                                                                     0xf, 0xf, false));
    };
    v += dpp(v, std::integral_constant<int, 0x111>{});
    v += dpp(v, std::integral_constant<int, 0x112>{});
    v += dpp(v, std::integral_constant<int, 0x114>{});
    v += dpp(v, std::integral_constant<int, 0x118>{});
    return v;
}

extern __shared__ __align__(16) float bw_lds[];

// ---------------------------------------------------------------------------
// S per tile.  A block takes a 64 x 32 pixel tile of one (image, channel) plane: grad_out's
// tile and x's zero-extended halo tile go to LDS.  Thread (tx, tg) = (t & 15, t >> 4) owns the
// 4-pixel column strip tx and two rows (2*ip, 2*ip + 1) of the correlation window; with at
// most eight row pairs the sixteen groups also split the tile's rows in two halves.  Walking
// down its rows it reads one grad_out segment and one new x segment per row (the x segment
// of window row 2*ip + 1 at tile row y is that of window row 2*ip at y + 1) and applies
// 2 * KC * 4 multiply-adds to its 2 * KC sums - the forward tap loop's ratio of arithmetic
// to LDS traffic.  The strip sums are added along each row of 16 lanes, then over the row
// halves, and written as the tile's partial sums; the last entry is the tile's sum of x
// (for the GAP).
// ---------------------------------------------------------------------------
template <typename T, int KC>
__global__ __launch_bounds__(kBwThreads) void corr_kernel(const BackwardParams p)
{
    constexpr int P = (KC - 1) / 2;
    constexpr int NP = (KC + 1) / 2;             // row pairs of the window
    constexpr int YS = NP <= 8 ? 2 : 1;           // halves the tile's rows are split in
    constexpr int ROWS = kCorrTileH / YS;
    constexpr int NXV = (KC + 3 + 3) & ~3;        // x values a thread reads per row
    constexpr int HC = kCorrTileW + KC - 1;
    constexpr int PITCH = ((60 + NXV > HC ? 60 + NXV : HC) + 3) & ~3;
    constexpr int HR = kCorrTileH + KC - 1 + 1;   // one spare row of zeros (an odd window's last pair reads it)
    float *xs = bw_lds;                            // [HR][PITCH]
    float *gs = xs + HR * PITCH;                   // [32][64]
    float *red = gs + kCorrTileH * kCorrTileW;     // [16][2*KC + 1]

    const int tid = (int)threadIdx.x;
    const int H = p.H, W = p.W;
    const int tiles_x = (W + kCorrTileW - 1) / kCorrTileW;
    const int tiles = corr_tiles(H, W);
    const unsigned nc = blockIdx.x / (unsigned)tiles, tile = blockIdx.x - nc * (unsigned)tiles;
    const unsigned n = nc / (unsigned)p.Ca, c = nc - n * (unsigned)p.Ca;
    const int ty0 = (int)(tile / (unsigned)tiles_x) * kCorrTileH, tx0 = (int)(tile % (unsigned)tiles_x) * kCorrTileW;
    const size_t plane = ((size_t)n * p.C + c) * (size_t)H * W;
    const T *xp = (const T *)p.x + plane, *gp = (const T *)p.go + plane;

    // ---- tiles to LDS (all of a batch's loads before their uses) ----
    for (int i0 = 0; i0 < HR * PITCH; i0 += 8 * kBwThreads) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int idx = i0 + u * kBwThreads + tid;
            const int r = idx / PITCH, cc = idx - r * PITCH;
            const int gy = ty0 - P + r, gx = tx0 - P + cc;
            const bool in = idx < HR * PITCH && gy >= 0 && gy < H && gx >= 0 && gx < W;
            v[u] = bw_load(xp + (in ? (size_t)gy * W + gx : 0));
            v[u] = in ? v[u] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int idx = i0 + u * kBwThreads + tid;
            if (idx < HR * PITCH) xs[idx] = v[u];
        }
    }
    {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int idx = u * kBwThreads + tid;
            const int r = idx >> 6, cc = idx & 63;
            const int gy = ty0 + r, gx = tx0 + cc;
            const bool in = gy < H && gx < W;
            v[u] = bw_load(gp + (in ? (size_t)gy * W + gx : 0));
            v[u] = in ? v[u] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) gs[u * kBwThreads + tid] = v[u];
    }
    __syncthreads();

    const int tx = tid & 15, tg = tid >> 4;
    const int ip = YS == 2 ? (tg & 7) : tg, yh = YS == 2 ? (tg >> 3) : 0;
    const int i_first = 2 * ip;
    float acc0[KC], acc1[KC];
#pragma unroll
    for (int j = 0; j < KC; ++j) acc0[j] = acc1[j] = 0.f;
    float sx = 0.f;
    if (i_first < KC) {  // (uniform per row of 16 lanes)
        const int ya = yh * ROWS;
        float xa[NXV], xb[NXV];
        {
            const float4 *src = reinterpret_cast<const float4 *>(xs + (ya + i_first) * PITCH + 4 * tx);
#pragma unroll
            for (int k = 0; k < NXV / 4; ++k) {
                const float4 f = src[k];
                xa[4 * k] = f.x, xa[4 * k + 1] = f.y, xa[4 * k + 2] = f.z, xa[4 * k + 3] = f.w;
            }
        }
        for (int y = ya; y < ya + ROWS; ++y) {
            const float4 g4 = *reinterpret_cast<const float4 *>(gs + y * kCorrTileW + 4 * tx);
            const float4 *src = reinterpret_cast<const float4 *>(xs + (y + i_first + 1) * PITCH + 4 * tx);
#pragma unroll
            for (int k = 0; k < NXV / 4; ++k) {
                const float4 f = src[k];
                xb[4 * k] = f.x, xb[4 * k + 1] = f.y, xb[4 * k + 2] = f.z, xb[4 * k + 3] = f.w;
            }
            const float g[4] = {g4.x, g4.y, g4.z, g4.w};
#pragma unroll
            for (int j = 0; j < KC; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    acc0[j] = fmaf(g[q], xa[q + j], acc0[j]);
                    acc1[j] = fmaf(g[q], xb[q + j], acc1[j]);
                }
            if (ip == 0) {  // the tile's own pixels, for the GAP: the window's centre row of this tile row
                const float *ctr = xs + (y + P) * PITCH + 4 * tx + P;
                sx += (ctr[0] + ctr[1]) + (ctr[2] + ctr[3]);
            }
#pragma unroll
            for (int k = 0; k < NXV; ++k) xa[k] = xb[k];
        }
    }
    // ---- strips -> rows of 16 lanes -> row halves -> the tile's partial sums ----
#pragma unroll
    for (int j = 0; j < KC; ++j) {
        const float a = row16_sum(acc0[j]), b = row16_sum(acc1[j]);
        if (tx == 15) {
            red[tg * (2 * KC + 1) + j] = a;
            red[tg * (2 * KC + 1) + KC + j] = b;
        }
    }
    {
        const float a = row16_sum(sx);
        if (tx == 15) red[tg * (2 * KC + 1) + 2 * KC] = a;
    }
    __syncthreads();
    float *dst = p.partial + ((size_t)nc * tiles + tile) * (KC * KC + 1);
    for (int o = tid; o < KC * KC + 1; o += kBwThreads) {
        float s;
        if (o == KC * KC) {
            s = red[2 * KC];
            if (YS == 2) s += red[8 * (2 * KC + 1) + 2 * KC];
        } else {
            const int i = o / KC, j = o - i * KC;
            const int g0 = i >> 1, off = (i & 1) * KC + j;
            s = red[g0 * (2 * KC + 1) + off];
            if (YS == 2) s += red[(g0 + 8) * (2 * KC + 1) + off];
        }
        dst[o] = s;
    }
}

// ---------------------------------------------------------------------------
// S per tile for windows up to 15 x 15, on the matrix cores.  For one row y of grad_out's
// tile the sums over x are a product of two 16 x K matrices:
//   S[i][j] += sum_c  X_y[i][c] * G_y[c][j],   X_y[i][c] = xz[y + i][c]  (rows of x's halo tile),
//                                              G_y[c][j] = go[y][c - j]  (a Toeplitz matrix of the row)
// with K = the halo tile's columns, 32 per v_mfma_f32_16x16x32_bf16: 3 instructions per tile
// row, 96 per tile, against 5400 vector multiply-adds per thread in corr_kernel.  With bf16
// storage the stored values are the operands (products exact, fp32 accumulation).  fp32 values
// are split into three bf16 terms each (8 + 8 + 8 mantissa bits, by truncation: exact but for
// values within 2^24 of the smallest normal number, whose third term loses denormal bits), kept
// as three tiles, and all nine products of terms are accumulated - every product is still
// exact, and nine times 96 instructions are still a fifth of the vector loop's time.
// A operand: lane (i, kg) reads 16 bytes of halo row y + i - the halo tile is laid out from the
// aligned column x0 - 8, so every read is aligned.  B operand: lane (j, kg) wants eight
// consecutive values of the row starting j elements to the left - a start that is odd for
// every other lane.  grad_out's rows are therefore kept twice, zero-extended: as they are and
// moved by one element; a lane reads four whole words from the copy of its parity.  The four
// wavefronts take eight rows each (neighbouring rows share their A operands, see there) and add
// their results through LDS; the sum of x (for the
// GAP) comes from the halo tile's loads.  Same partial sums, same layout as corr_kernel.
// ---------------------------------------------------------------------------
constexpr int kCmXP = 104;  // halo tile: elements per row (96 columns are read; 13 x 16 bytes: rows fall on different banks)
constexpr int kCmXR = 48;   // halo tile rows (rows up to 31 + 15 are read; those beyond the window feed discarded results)
constexpr int kCmGP = 112;  // elements per zero-extended row of grad_out
constexpr size_t kCmG0 = (size_t)kCmXR * kCmXP * 2, kCmG1 = kCmG0 + (size_t)kCorrTileH * kCmGP * 2 + 64;
constexpr size_t kCmLds = kCmG1 + (size_t)kCorrTileH * kCmGP * 2;  // per term

// eight consecutive bf16 values to row[q ...]: whole words where the parity of q allows
template <bool EVEN>
__device__ __forceinline__ void cm_put8(uint16_t *row, int q, const uint16_t (&v)[8])
{
    if (EVEN) {
#pragma unroll
        for (int d = 0; d < 4; ++d) *reinterpret_cast<uint32_t *>(row + q + 2 * d) = (uint32_t)v[2 * d] | ((uint32_t)v[2 * d + 1] << 16);
    } else {
        row[q] = v[0];
#pragma unroll
        for (int d = 0; d < 3; ++d) *reinterpret_cast<uint32_t *>(row + q + 1 + 2 * d) = (uint32_t)v[2 * d + 1] | ((uint32_t)v[2 * d + 2] << 16);
        row[q + 7] = v[7];
    }
}

template <typename T, int KC>
__global__ __launch_bounds__(kBwThreads) void corr_mfma_kernel(const BackwardParams p)
{
    typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    static_assert(KC % 2 == 1 && KC >= 3 && KC <= 15, "one 16 x 16 block of sums");
    constexpr bool kF32 = std::is_same<T, float>::value;
    constexpr int NT = kF32 ? 3 : 1;          // bf16 terms per value
    constexpr int P = (KC - 1) / 2;
    constexpr int HRU = kCorrTileH + KC - 1;  // halo rows the window reaches
    constexpr int GOFF = P + 8;               // element of a zero-extended row that holds the tile's column 0
    char *lds = reinterpret_cast<char *>(bw_lds);
    // term t: halo tile [kCmXR][kCmXP] (column c = image column x0 - 8 + c), then grad_out's rows
    // [32][kCmGP] (element q = column q - GOFF) and the same moved by one (element q = column q + 1 - GOFF)
    auto xs = [&](int t) { return reinterpret_cast<uint16_t *>(lds + t * kCmLds); };
    auto g0 = [&](int t) { return reinterpret_cast<uint16_t *>(lds + t * kCmLds + kCmG0); };
    auto g1 = [&](int t) { return reinterpret_cast<uint16_t *>(lds + t * kCmLds + kCmG1); };

    const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int H = p.H, W = p.W;
    const int tiles_x = (W + kCorrTileW - 1) / kCorrTileW;
    const int tiles = corr_tiles(H, W);
    const unsigned nc = blockIdx.x / (unsigned)tiles, tile = blockIdx.x - nc * (unsigned)tiles;
    const unsigned n = nc / (unsigned)p.Ca, c = nc - n * (unsigned)p.Ca;
    const int ty0 = (int)(tile / (unsigned)tiles_x) * kCorrTileH, tx0 = (int)(tile % (unsigned)tiles_x) * kCorrTileW;
    const size_t plane = ((size_t)n * p.C + c) * (size_t)H * W;
    const T *xp = (const T *)p.x + plane, *gp = (const T *)p.go + plane;

    // a value as NT bf16 terms (fp32: the top eight mantissa bits, the next eight, the rest - exact)
    auto split = [](float v, uint16_t (&t)[3]) {
        const uint32_t hb = __float_as_uint(v) & 0xffff0000u;
        const float r1 = v - __uint_as_float(hb);
        const uint32_t mb = __float_as_uint(r1) & 0xffff0000u;
        const float r2 = r1 - __uint_as_float(mb);
        t[0] = (uint16_t)(hb >> 16), t[1] = (uint16_t)(mb >> 16), t[2] = (uint16_t)(__float_as_uint(r2) >> 16);
    };
    // eight neighbouring values (16 or 32 bytes of memory) at e, or zeros; their sum for the GAP
    auto fetch8 = [](const T *e, bool in, u32x4 (&raw)[kF32 ? 2 : 1]) {
        raw[0] = *reinterpret_cast<const u32x4 *>(e);
        if (kF32) raw[kF32 ? 1 : 0] = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(e) + 16);
        if (!in)
            for (int k = 0; k < (kF32 ? 2 : 1); ++k) raw[k] = u32x4{0u, 0u, 0u, 0u};
    };
    auto terms8 = [&](const u32x4 (&raw)[kF32 ? 2 : 1], uint16_t (&v)[NT][8], float &sum) {
        sum = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (kF32) {
                uint16_t t3[3];
                const float f = __uint_as_float(raw[kF32 ? e >> 2 : 0][e & 3]);
                split(f, t3);
#pragma unroll
                for (int t = 0; t < NT; ++t) v[t][e] = t3[t];
                sum += f;
            } else {
                v[0][e] = (uint16_t)(raw[0][e >> 1] >> (16 * (e & 1)));
                sum += __uint_as_float((uint32_t)v[0][e] << 16);
            }
        }
    };

    float sx = 0.f;
    if (p.corr_vec) {
        // whole pieces of eight columns, each entirely inside or outside the image; the loads
        // travel while the LDS is cleared
        constexpr int XT = HRU * 10, XK = (XT + kBwThreads - 1) / kBwThreads;
        u32x4 xv[XK][kF32 ? 2 : 1], gv[kF32 ? 2 : 1];
#pragma unroll
        for (int k = 0; k < XK; ++k) {
            const int t = k * kBwThreads + tid, r = t / 10, pc = t - r * 10;
            const int gy = ty0 - P + r, gx = tx0 - 8 + 8 * pc;
            const bool in = t < XT && gy >= 0 && gy < H && gx >= 0 && gx < W;
            fetch8(xp + (in ? (size_t)gy * W + gx : 0), in, xv[k]);
        }
        {
            const int r = tid >> 3, pc = tid & 7;
            const int gy = ty0 + r, gx = tx0 + 8 * pc;
            const bool in = gy < H && gx < W;
            fetch8(gp + (in ? (size_t)gy * W + gx : 0), in, gv);
        }
        for (int o = tid; o < (int)(NT * kCmLds / 16); o += kBwThreads) reinterpret_cast<u32x4 *>(lds)[o] = u32x4{0u, 0u, 0u, 0u};
        __syncthreads();
#pragma unroll
        for (int k = 0; k < XK; ++k) {
            const int t = k * kBwThreads + tid, r = t / 10, pc = t - r * 10;
            uint16_t v[NT][8];
            float sum;
            terms8(xv[k], v, sum);
            if (t < XT) {
#pragma unroll
                for (int tt = 0; tt < NT; ++tt) cm_put8<true>(xs(tt) + r * kCmXP, 8 * pc, v[tt]);
                // the tile's own pixels, for the GAP
                if (r >= P && r < P + kCorrTileH && pc >= 1 && pc <= 8) sx += sum;
            }
        }
        {
            const int r = tid >> 3, pc = tid & 7;
            uint16_t v[NT][8];
            float sum;
            terms8(gv, v, sum);
#pragma unroll
            for (int tt = 0; tt < NT; ++tt) {
                cm_put8<GOFF % 2 == 0>(g0(tt) + r * kCmGP, GOFF + 8 * pc, v[tt]);
                cm_put8<GOFF % 2 != 0>(g1(tt) + r * kCmGP, GOFF + 8 * pc - 1, v[tt]);
            }
        }
    } else {
        for (int o = tid; o < (int)(NT * kCmLds / 16); o += kBwThreads) reinterpret_cast<u32x4 *>(lds)[o] = u32x4{0u, 0u, 0u, 0u};
        __syncthreads();
        for (int t = tid; t < HRU * 80; t += kBwThreads) {
            const int r = t / 80, cc = t - r * 80;
            const int gy = ty0 - P + r, gx = tx0 - 8 + cc;
            if (gy >= 0 && gy < H && gx >= 0 && gx < W) {
                const float f = bw_load(xp + (size_t)gy * W + gx);
                uint16_t t3[3];
                split(f, t3);
#pragma unroll
                for (int tt = 0; tt < NT; ++tt) xs(tt)[r * kCmXP + cc] = t3[tt];
                if (r >= P && r < P + kCorrTileH && cc >= 8 && cc < 8 + kCorrTileW) sx += f;
            }
        }
        for (int t = tid; t < kCorrTileH * kCorrTileW; t += kBwThreads) {
            const int r = t >> 6, cc = t & 63;
            const int gy = ty0 + r, gx = tx0 + cc;
            if (gy < H && gx < W) {
                uint16_t t3[3];
                split(bw_load(gp + (size_t)gy * W + gx), t3);
#pragma unroll
                for (int tt = 0; tt < NT; ++tt) {
                    g0(tt)[r * kCmGP + GOFF + cc] = t3[tt];
                    g1(tt)[r * kCmGP + GOFF + cc - 1] = t3[tt];
                }
            }
        }
    }
    __syncthreads();

    // ---- this wavefront's rows of the tile: 8 w .. 8 w + 7, in groups of SH neighbours that
    // share their A operands: the halo rows R .. R + 15 serve tile row R + s as window rows
    // i = i' - s (i' the row of the product), s < SH = 16 - KC + 1 (at most 4); every shift has
    // accumulators of its own, and the shifted results are put together at the end ----
    constexpr int SH = KC <= 13 ? 4 : 2;
    const int l16 = lane & 15, kg = lane >> 4;
    const int jc = l16 < KC ? l16 : KC - 1;  // (columns beyond the window repeat its last one; their sums are dropped)
    const size_t gsel = (jc & 1) ? kCmG1 : kCmG0;
    const int o0 = 8 * kg - jc + 2 * P - (jc & 1);  // even: the lane's first element in its copy, for block 0
    f32x4 acc[SH][3];
#pragma unroll
    for (int sft = 0; sft < SH; ++sft)
#pragma unroll
        for (int b = 0; b < 3; ++b) acc[sft][b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < 8 / SH; ++u) {
        const int R = 8 * wave + SH * u;
        u32x4 a[NT][3];
#pragma unroll
        for (int tt = 0; tt < NT; ++tt)
#pragma unroll
            for (int b = 0; b < 3; ++b) a[tt][b] = *reinterpret_cast<const u32x4 *>(xs(tt) + (R + l16) * kCmXP + 32 * b + 8 * kg);
#pragma unroll
        for (int sft = 0; sft < SH; ++sft) {
            u32x4 bv[NT][3];
#pragma unroll
            for (int tt = 0; tt < NT; ++tt)
#pragma unroll
                for (int b = 0; b < 3; ++b)
                    __builtin_memcpy(&bv[tt][b],
                                     reinterpret_cast<const uint32_t *>(reinterpret_cast<const uint16_t *>(lds + tt * kCmLds + gsel) +
                                                                        (R + sft) * kCmGP + o0 + 32 * b),
                                     16);
            // (small terms first; the three column blocks' chains take turns)
#pragma unroll
            for (int ta = NT - 1; ta >= 0; --ta)
#pragma unroll
                for (int tb = NT - 1; tb >= 0; --tb)
#pragma unroll
                    for (int b = 0; b < 3; ++b)
                        acc[sft][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[ta][b]),
                                                                              __builtin_bit_cast(bf16x8, bv[tb][b]), acc[sft][b], 0, 0, 0);
        }
    }
    const float sxr = row16_sum(sx);
    __syncthreads();  // the tiles are no longer read: their LDS takes the wavefronts' results
    float *red = bw_lds;                   // [4 wavefronts][SH shifts][16 i'][16 j]
    float *sxs = bw_lds + 4 * SH * 256;    // [16 rows of lanes]
#pragma unroll
    for (int sft = 0; sft < SH; ++sft) {
        const f32x4 tot = (acc[sft][0] + acc[sft][1]) + acc[sft][2];
#pragma unroll
        for (int r = 0; r < 4; ++r) red[(wave * SH + sft) * 256 + (4 * kg + r) * 16 + l16] = tot[r];
    }
    if (l16 == 15) sxs[tid >> 4] = sxr;
    __syncthreads();
    float *dst = p.partial + ((size_t)nc * tiles + tile) * (KC * KC + 1);
    for (int o = tid; o < KC * KC + 1; o += kBwThreads) {
        float s2 = 0.f;
        if (o == KC * KC) {
#pragma unroll
            for (int k = 0; k < 16; ++k) s2 += sxs[k];
        } else {
            const int i = o / KC, j = o - i * KC;
#pragma unroll
            for (int w = 0; w < 4; ++w)
#pragma unroll
                for (int sft = 0; sft < SH; ++sft) s2 += red[(w * SH + sft) * 256 + (i + sft) * 16 + j];
        }
        dst[o] = s2;
    }
}

template <typename T, int KC>
hipError_t launch_corr_mfma(const BackwardParams &p, unsigned grid, hipStream_t s)
{
    constexpr size_t lds = (std::is_same<T, float>::value ? 3 : 1) * kCmLds;
    static bool granted = false;
    if (lds > 48 * 1024 && !granted) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&corr_mfma_kernel<T, KC>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        granted = true;
    }
    hipLaunchKernelGGL((corr_mfma_kernel<T, KC>), dim3(grid), dim3(kBwThreads), lds, s, p);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_corr_mfma_kc(const BackwardParams &p, int kc, unsigned grid, hipStream_t s)
{
    switch (kc) {
#define ESC_KC(K) case K: return launch_corr_mfma<T, K>(p, grid, s);
        ESC_KC(3) ESC_KC(5) ESC_KC(7) ESC_KC(9) ESC_KC(11) ESC_KC(13) ESC_KC(15)
#undef ESC_KC
    }
    return hipErrorInvalidValue;
}

// grad_lk: one row of 16 lanes per element (element idx of the Ks x Ks filters; sums over images
// and tiles, over channels too for a single shared filter).  Lane l adds terms l, l + 16, ...
// in ascending order, then the row's lanes are added in lane order: a fixed order, and
// sixteen loads in flight instead of a chain of dependent ones.
__device__ __forceinline__ void sums_row(const BackwardParams &p, int KC, int tiles, size_t idx, int l)
{
    const int Ks = p.Ks, Ca = p.Ca, off = (KC - Ks) / 2;
    const size_t per = (size_t)KC * KC + 1;
    const int c0 = (int)(idx / ((size_t)Ks * Ks)), r = (int)(idx % ((size_t)Ks * Ks));
    const size_t elem = (size_t)(r / Ks + off) * KC + (size_t)(r % Ks + off);
    // channel c0 of every image, or (one shared filter) every channel of every image
    const size_t nc0 = p.lk_cstride != 0 ? (size_t)c0 : 0;
    const int planes = p.lk_cstride != 0 ? p.N : p.N * Ca, plane_step = p.lk_cstride != 0 ? Ca : 1;
    const int count = planes * tiles;
    float s = 0.f;
    for (int k0 = l; k0 < count; k0 += 64) {
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int k = k0 + 16 * u;
            const int kk = k < count ? k : count - 1;
            const int pl = kk / tiles, tl = kk - pl * tiles;
            v[u] = p.partial[((nc0 + (size_t)pl * plane_step) * tiles + tl) * per + elem];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) s += k0 + 16 * u < count ? v[u] : 0.f;
    }
    s = row16_sum(s);
    if (l != 15 || p.grad_lk == nullptr) return;
    float *dst = p.grad_lk + (p.lk_cstride != 0 ? (size_t)c0 * p.lk_cstride : 0) + r;
    *dst = p.accumulate ? *dst + s : s;
}

__device__ __forceinline__ float gelu_f(float v) { return 0.5f * v * (1.f + erff(v * 0.70710678118654752440f)); }
__device__ __forceinline__ float gelu_grad_f(float v)
{
    return 0.5f * (1.f + erff(v * 0.70710678118654752440f)) + v * expf(-0.5f * v * v) * 0.39894228040143267794f;
}

// One block per image: its tiles' partial sums are added to dDK[n] and the GAP means g[n]
// (a thread per result); then the estimator forwards from g (DK, stored flipped for the input
// gradient) and backwards from dDK (dL/dt, dL/du, dL/dg) - plain loops, a few thousand
// multiply-adds per image.
__global__ __launch_bounds__(kBwThreads) void estimator_image_kernel(const BackwardParams p, int KC, int tiles)
{
    __shared__ float s_g[256], s_u[256], s_t[256], s_dt[256], s_du[256], s_dd[9 * 256], s_part[kBwThreads];
    const int n = (int)blockIdx.x, tid = (int)threadIdx.x;
    const int Ca = p.Ca, hidden = p.hidden, K = hidden > 0 ? hidden : Ca;
    const float hw = (float)((double)p.H * (double)p.W);
    {
        // this image's sums over its tiles, one thread per result (9 C_a of dDK, C_a of g), the
        // tiles in ascending order, eight loads in flight
        const size_t per = (size_t)KC * KC + 1;
        for (int o = tid; o < 10 * Ca; o += kBwThreads) {
            const bool is_dd = o < 9 * Ca;
            const int c = is_dd ? o / 9 : o - 9 * Ca, r = is_dd ? o - 9 * c : 0;
            const size_t elem = is_dd ? (size_t)(r / 3 + (KC - 3) / 2) * KC + (size_t)(r % 3 + (KC - 3) / 2) : (size_t)KC * KC;
            const float *src = p.partial + ((size_t)n * Ca + c) * tiles * per + elem;
            float sum = 0.f;
            for (int t0 = 0; t0 < tiles; t0 += 8) {
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = src[(size_t)(t0 + u < tiles ? t0 + u : tiles - 1) * per];
#pragma unroll
                for (int u = 0; u < 8; ++u) sum += t0 + u < tiles ? v[u] : 0.f;
            }
            if (is_dd) {
                s_dd[o] = sum;
                p.ddk[(size_t)n * 9 * Ca + o] = sum;
                if (p.grad_dk != nullptr) p.grad_dk[(size_t)n * 9 * Ca + o] = sum;
            } else {
                const float g = sum / hw;
                s_g[c] = g;
                p.g[(size_t)n * Ca + c] = g;
            }
        }
    }
    if (!p.has_gen) {  // DK as given (or zero): only its flipped copy is needed
        for (int o = tid; o < 9 * Ca; o += kBwThreads) {
            const int c = o / 9, r = o - 9 * c;
            p.dkf[((size_t)n * Ca + c) * 9 + (8 - r)] = p.dk_in != nullptr ? p.dk_in[(size_t)n * 9 * Ca + o] : 0.f;
        }
        for (int k = tid; k < Ca; k += kBwThreads) p.dgc[(size_t)n * Ca + k] = 0.f;
        return;
    }
    __syncthreads();  // s_g and s_dd are written
    if (hidden > 0) {
        for (int m = tid; m < hidden; m += kBwThreads) {
            float s = p.b_down != nullptr ? p.b_down[m] : 0.f;
#pragma unroll 8
            for (int k = 0; k < Ca; ++k) s = fmaf(p.w_down[(size_t)m * Ca + k], s_g[k], s);
            s_u[m] = s;
            s_t[m] = gelu_f(s);
        }
    } else {
        for (int k = tid; k < Ca; k += kBwThreads) s_t[k] = s_g[k];
    }
    __syncthreads();
    for (int k = tid; k < K; k += kBwThreads) p.t[(size_t)n * K + k] = s_t[k];
    for (int o = tid; o < 9 * Ca; o += kBwThreads) {
        float s = p.b_up != nullptr ? p.b_up[o] : 0.f;
#pragma unroll 8
        for (int k = 0; k < K; ++k) s = fmaf(p.w_up[(size_t)o * K + k], s_t[k], s);
        const int c = o / 9, r = o - 9 * c;
        p.dkf[((size_t)n * Ca + c) * 9 + (8 - r)] = s;
    }
    // dL/dt = w_up^T dd: the rows o are dealt to the block's groups of K threads (group g takes
    // rows g, g + groups, ...), whose partial sums are then added in group order - a chain of
    // 9 C_a dependent loads per thread otherwise
    if (K <= kBwThreads / 2) {
        const int groups = kBwThreads / K, g = tid / K, k = tid - g * K;
        float s = 0.f;
        if (g < groups) {
#pragma unroll 4
            for (int o = g; o < 9 * Ca; o += groups) s = fmaf(p.w_up[(size_t)o * K + k], s_dd[o], s);
            s_part[g * K + k] = s;
        }
        __syncthreads();
        if (tid < K) {
            float t = 0.f;
            for (int q = 0; q < groups; ++q) t += s_part[q * K + tid];
            s_dt[tid] = t;
        }
    } else {
        for (int k = tid; k < K; k += kBwThreads) {
            float s = 0.f;
#pragma unroll 8
            for (int o = 0; o < 9 * Ca; ++o) s = fmaf(p.w_up[(size_t)o * K + k], s_dd[o], s);
            s_dt[k] = s;
        }
    }
    __syncthreads();
    if (hidden > 0) {
        for (int m = tid; m < hidden; m += kBwThreads) {
            const float v = s_dt[m] * gelu_grad_f(s_u[m]);
            s_du[m] = v;
            p.du[(size_t)n * hidden + m] = v;
        }
        __syncthreads();
        for (int k = tid; k < Ca; k += kBwThreads) {
            float s = 0.f;
#pragma unroll 8
            for (int m = 0; m < hidden; ++m) s = fmaf(p.w_down[(size_t)m * Ca + k], s_du[m], s);
            p.dgc[(size_t)n * Ca + k] = s / hw;
        }
    } else {
        for (int k = tid; k < Ca; k += kBwThreads) p.dgc[(size_t)n * Ca + k] = s_dt[k] / hw;
    }
}

// One row of 16 lanes per result of the sums over the batch: grad_lk (sums_row) and the
// estimator's parameters (lane l adds images l, l + 16, ... in ascending order, then the
// row's lanes in lane order); the flipped LK takes one lane per element behind them.
__global__ __launch_bounds__(256) void batch_sums_kernel(const BackwardParams p, int KC, int tiles)
{
    const int Ca = p.Ca, hidden = p.hidden, K = hidden > 0 ? hidden : Ca, Ks = p.Ks;
    const size_t n_lk = (size_t)(p.lk_cstride != 0 ? Ca : 1) * Ks * Ks;
    const size_t n_wu = p.has_gen ? (size_t)9 * Ca * K : 0, n_bu = p.has_gen ? (size_t)9 * Ca : 0;
    const size_t n_wd = p.has_gen ? (size_t)hidden * Ca : 0, n_bd = p.has_gen ? (size_t)hidden : 0;
    size_t idx = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 4;  // uniform per row of 16 lanes
    const int l = (int)(threadIdx.x & 15);
    if (idx < n_lk) {
        sums_row(p, KC, tiles, idx, l);
        return;
    }
    idx -= n_lk;
    if (idx >= n_wu + n_bu + n_wd + n_bd) {  // the flipped large kernel: one element per lane of the rows left over
        const size_t e = (idx - (n_wu + n_bu + n_wd + n_bd)) * 16 + l;
        if (e < n_lk) {
            const size_t c = e / ((size_t)Ks * Ks), r = e % ((size_t)Ks * Ks);
            p.lkf[e] = p.lk[c * (size_t)p.lk_cstride + ((size_t)Ks * Ks - 1 - r)];
        }
        return;
    }
    // result = sum_n a[n * sa + ia] * b[n * sb + ib]   (b == nullptr: the plain sum of a)
    const float *a, *b = nullptr;
    size_t sa, ia, sb = 0, ib = 0;
    float *dst;
    if (idx < n_wu) {
        a = p.ddk, sa = (size_t)9 * Ca, ia = idx / K;
        b = p.t, sb = (size_t)K, ib = idx % K;
        dst = p.grad_w_up ? p.grad_w_up + idx : nullptr;
    } else if ((idx -= n_wu) < n_bu) {
        a = p.ddk, sa = (size_t)9 * Ca, ia = idx;
        dst = p.grad_b_up ? p.grad_b_up + idx : nullptr;
    } else if ((idx -= n_bu) < n_wd) {
        a = p.du, sa = (size_t)hidden, ia = idx / Ca;
        b = p.g, sb = (size_t)Ca, ib = idx % Ca;
        dst = p.grad_w_down ? p.grad_w_down + idx : nullptr;
    } else {
        idx -= n_wd;
        a = p.du, sa = (size_t)hidden, ia = idx;
        dst = p.grad_b_down ? p.grad_b_down + idx : nullptr;
    }
    float s = 0.f;
    for (int n = l; n < p.N; n += 16) s = b != nullptr ? fmaf(a[(size_t)n * sa + ia], b[(size_t)n * sb + ib], s) : s + a[(size_t)n * sa + ia];
    s = row16_sum(s);
    if (l == 15 && dst != nullptr) *dst = p.accumulate ? *dst + s : s;
}


template <typename T, int KC>
hipError_t launch_corr(const BackwardParams &p, unsigned grid, hipStream_t s)
{
    constexpr int NXV = (KC + 3 + 3) & ~3, HC = kCorrTileW + KC - 1;
    constexpr int PITCH = ((60 + NXV > HC ? 60 + NXV : HC) + 3) & ~3, HR = kCorrTileH + KC;
    constexpr size_t lds = ((size_t)HR * PITCH + kCorrTileH * kCorrTileW + 16 * (2 * KC + 1)) * sizeof(float);
    static_assert(lds <= 64 * 1024, "the correlation kernel's tiles must fit the default LDS limit");
    hipLaunchKernelGGL((corr_kernel<T, KC>), dim3(grid), dim3(kBwThreads), lds, s, p);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_corr_kc(const BackwardParams &p, int kc, unsigned grid, hipStream_t s)
{
    switch (kc) {
#define ESC_KC(K) case K: return launch_corr<T, K>(p, grid, s);
        ESC_KC(3) ESC_KC(5) ESC_KC(7) ESC_KC(9) ESC_KC(11) ESC_KC(13) ESC_KC(15) ESC_KC(17)
        ESC_KC(19) ESC_KC(21) ESC_KC(23) ESC_KC(25) ESC_KC(27) ESC_KC(29) ESC_KC(31)
#undef ESC_KC
    }
    return hipErrorInvalidValue;
}

}  // namespace

// the correlation of grad_out with x, tile by tile
__attribute__((visibility("hidden"))) hipError_t launch_backward_sums(const BackwardParams &p, bool bf16, hipStream_t s)
{
    if (p.Ca < 1) return hipSuccess;
    const int kc = corr_window(p.Ks), tiles = corr_tiles(p.H, p.W);
    const size_t grid = (size_t)p.N * p.Ca * tiles;
    if (grid >= ((size_t)1 << 31)) return hipErrorInvalidValue;
    if (kc <= 15) {  // one 16 x 16 block of sums: the matrix cores
        BackwardParams q = p;
        q.corr_vec = (p.W % 8 == 0) && ((uintptr_t)p.x % 16 == 0) && ((uintptr_t)p.go % 16 == 0);
        return bf16 ? launch_corr_mfma_kc<bf16b>(q, kc, (unsigned)grid, s) : launch_corr_mfma_kc<float>(q, kc, (unsigned)grid, s);
    }
    return bf16 ? launch_corr_kc<bf16b>(p, kc, (unsigned)grid, s) : launch_corr_kc<float>(p, kc, (unsigned)grid, s);
}

// per image: dDK and g from the tiles' sums, the estimator forwards and backwards, the
// flipped kernels (all that the input gradient's launch needs); then the sums over the
// batch: grad_lk and the estimator's parameter gradients
__attribute__((visibility("hidden"))) hipError_t launch_backward_estimator(const BackwardParams &p, hipStream_t s)
{
    if (p.Ca < 1) return hipSuccess;
    const int kc = corr_window(p.Ks), tiles = corr_tiles(p.H, p.W);
    hipLaunchKernelGGL(estimator_image_kernel, dim3((unsigned)p.N), dim3(kBwThreads), 0, s, p, kc, tiles);
    return hipGetLastError();
}

__attribute__((visibility("hidden"))) hipError_t launch_backward_batch_sums(const BackwardParams &p, hipStream_t s)
{
    if (p.Ca < 1) return hipSuccess;
    const int kc = corr_window(p.Ks), tiles = corr_tiles(p.H, p.W);
    const size_t K = p.hidden > 0 ? (size_t)p.hidden : (size_t)p.Ca;
    const size_t rows = (size_t)(p.lk_cstride != 0 ? p.Ca : 1) * p.Ks * p.Ks +
                        (p.has_gen ? (size_t)9 * p.Ca * K + 9 * p.Ca + (size_t)p.hidden * p.Ca + p.hidden : 0);
    const size_t n_lkf = (size_t)(p.lk_cstride != 0 ? p.Ca : 1) * p.Ks * p.Ks;  // one lane per element behind the rows
    hipLaunchKernelGGL(batch_sums_kernel, dim3((unsigned)((rows * 16 + n_lkf + 255) / 256)), dim3(256), 0, s, p, kc, tiles);
    return hipGetLastError();
}

}  // namespace esc

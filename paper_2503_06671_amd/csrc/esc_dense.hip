// The ConvAttn module with the DENSE large kernel of the ESC paper's main variants
// (Sec. 3: LK in R^{Ks x Ks x C_a x C_a}, shared by the whole model; Eq. 4 line 3
//   F_res = F_att (*) DK + F_att (*) LK,  DK depth-wise, kept unmerged as the paper does)
// for gfx950 (MI355X).
//
// A full C_a -> C_a convolution is a dense contraction over K = C_a * Ks * Ks (2704 for the
// paper's 13 x 13 x 16 x 16), sixteen times the depth-wise form's arithmetic on the same
// bytes: it is bound by the matrix cores, so it runs as an implicit GEMM - with up to 16
// channels on the bf16 instructions (dense_bf16_kernel, further down: bf16 storage, and fp32
// storage up to 13 x 13 with values and weights as exact bf16 terms), else on
// v_mfma_f32_16x16x4_f32 (fp32 products and accumulation; bf16 storage is widened exactly
// when a tile is staged and rounded once at the store).  That kernel: per block an 8 x 32 (small calls:
// 4 x 32) pixel output tile of one image, all output channels.  Sixteen input channels at a time, their
// zero-extended halo tile sits in LDS; per kernel row the weights of its Ks taps
// ([tap][16 co][16 ci], rearranged once per call by a small kernel so that a row is one run
// of memory) are staged beside it, the next row's already in flight in registers.  Per tap
// and group of four input channels a wavefront reads one A operand per 16 output channels
// (lane l: W[co = l % 16][ci = l / 16]) and its B operands (lane l: pixel l % 16 of input
// channel l / 16, shifted by the tap - the im2col happens in the LDS address).  With more
// than 16 channels a wavefront owns a quarter of the tile's runs of 16 pixels and walks all
// input channels; with up to 16 (the paper's C_a) it owns four input channels - the K of one
// instruction - for all of the tile's runs, and the four partial results are added through
// LDS: eight to sixteen independent accumulators per wavefront instead of two, operands of
// the next tap in flight while this tap's instructions issue.  DK's nine depth-wise taps are
// added from the same tile on the vector units; the block also moves its share of the
// pass-through channels (Eq. 4 lines 1 and 4).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "esc_dense.hpp"
#include "esc_dense_weights.hpp"

namespace esc {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int kDnThreads = 256;
constexpr int kDnTw = 32;  // output tile width; its height TH is 8, or 4 when that is needed to fill the chip
constexpr unsigned kXcds = 8;

struct bf16d {
    uint16_t bits;
};
__device__ __forceinline__ float dn_load(const float *p) { return *p; }
__device__ __forceinline__ float dn_load(const bf16d *p) { return __uint_as_float((uint32_t)p->bits << 16); }
__device__ __forceinline__ uint16_t dn_f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ void dn_store(float *p, float v) { __builtin_nontemporal_store(v, p); }
__device__ __forceinline__ void dn_store(bf16d *p, float v) { __builtin_nontemporal_store(dn_f32_to_bf16(v), &p->bits); }

// halo tile geometry for a kernel size: rows, pitch and floats per channel plane (the plane
// stride is 16 modulo 32 banks, so the four channels of a B operand fall on both bank halves)
__host__ __device__ inline void dense_geom(int Ks, int th, int &hr, int &pitch, int &plane)
{
    const int p = (Ks - 1) / 2;
    hr = th + 2 * p;
    pitch = kDnTw + 2 * p;
    plane = hr * pitch;
    plane += (16 - plane % 32 + 32) % 32;
}

// wt[chunk][i][j][ct][ci][co] = lk[16 ct + co][16 chunk + ci][i - off][j - off], zero beyond C_a
// and outside the Ks x Ks kernel: the kernel is embedded, centred, in a Kse x Kse one (Kse =
// max(Ks, 3): the halo tile must also hold DK's 3 x 3 neighbourhood)
__global__ void dense_weights_kernel(const float *lk, int Ca, int Ks, int Kse, float *wt, size_t total)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int CT = (Ca + 15) / 16, off = (Kse - Ks) / 2;
    size_t r = idx;
    const int co = (int)(r % 16); r /= 16;
    const int ci = (int)(r % 16); r /= 16;
    const int ct = (int)(r % CT); r /= CT;
    const int j = (int)(r % Kse) - off; r /= Kse;
    const int i = (int)(r % Kse) - off; r /= Kse;
    const int chunk = (int)r;
    const int o = 16 * ct + co, c = 16 * chunk + ci;
    const bool in = o < Ca && c < Ca && i >= 0 && i < Ks && j >= 0 && j < Ks;
    wt[idx] = in ? lk[(((size_t)o * Ca + c) * Ks + i) * Ks + j] : 0.f;
}

extern __shared__ __align__(16) float dn_lds[];

// x / d for x < 2^31 by multiply-high and shift (dn_make_div fills mul and shift on the host)
__device__ __forceinline__ unsigned dn_div(unsigned x, unsigned mul, unsigned shift) { return (__umulhi(x, mul) + x) >> shift; }
void dn_make_div(unsigned d, unsigned &mul, unsigned &shift)
{
    unsigned l = 0;
    while (((uint64_t)1 << l) < d) ++l;
    mul = (unsigned)((((uint64_t)1 << 32) * (((uint64_t)1 << l) - d)) / d + 1);
    shift = l;
}

template <typename T, int CT, int TH>
__global__ __launch_bounds__(kDnThreads, CT <= 2 ? 2 : 1) void dense_kernel(const DenseParams p)
{
    constexpr int NT = TH / 2;  // runs of 16 pixels per wavefront: rows (TH/4)*wave .., two halves each
    constexpr int RW = TH / 4;
    const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, kq = lane >> 4;  // pixel (or output channel) within a run; input channel within a group of four
    const int Ks = p.Ks, pad = (Ks - 1) / 2, H = p.H, W = p.W;
    int HR, PITCH, PLANE;
    dense_geom(Ks, TH, HR, PITCH, PLANE);
    float *s_tile = dn_lds;                 // [16][PLANE]
    float *s_w = dn_lds + 16 * PLANE;       // [Ks][CT][16 ci][16 co]
    const int row_floats = Ks * CT * 256;

    // Blocks go to the chip's eight dies round robin; each die gets a contiguous eighth of the
    // tiles, so that neighbouring tiles (shared halos) meet in one L2.
    const unsigned nblk = gridDim.x, die = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
    const unsigned q = nblk / kXcds, rem = nblk % kXcds;
    const unsigned tile_id = die * q + (die < rem ? die : rem) + slot;
    const unsigned per_img = (unsigned)(p.tiles_x * p.tiles_y);
    const unsigned n = tile_id / per_img, t_in = tile_id - n * per_img;
    const int tyi = (int)(t_in / (unsigned)p.tiles_x), txi = (int)(t_in - (unsigned)tyi * p.tiles_x);
    const int y0 = tyi * TH, x0 = txi * kDnTw;
    const size_t plane_px = (size_t)H * W;
    const T *xn = (const T *)p.x + (size_t)n * p.C * plane_px;

    // ---- the block's share of the pass-through copy (Eq. 4 lines 1 and 4): issued first, it
    // streams while the first tile and weights arrive; its last 16 KiB round is stored only
    // behind the tile's loads (copy_last_store), so that the two round trips overlap ----
    u32x4 copy_v[4] = {};
    size_t copy_o0 = 0, copy_end = 0;
    char *copy_dst = nullptr;
    if (p.idt_len > 0) {
        const char *src = (const char *)p.x + (size_t)n * p.img_bytes + p.idt_off;
        char *dst = (char *)p.out + (size_t)n * p.img_bytes + p.idt_off;
        const size_t begin = (size_t)t_in * p.copy_share;
        const size_t end = begin + p.copy_share < p.idt_len ? begin + p.copy_share : p.idt_len;
        if (p.copy_vec) {
            constexpr size_t kRound = (size_t)4 * kDnThreads * 16;
            for (size_t o0 = begin; o0 < end; o0 += kRound) {
                u32x4 v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const size_t o = o0 + ((size_t)u * kDnThreads + tid) * 16;
                    v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + (o + 16 <= end ? o : begin)));
                }
                if (o0 + kRound >= end) {  // the last round (block-uniform)
#pragma unroll
                    for (int u = 0; u < 4; ++u) copy_v[u] = v[u];
                    copy_o0 = o0, copy_end = end, copy_dst = dst;
                    break;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const size_t o = o0 + ((size_t)u * kDnThreads + tid) * 16;
                    if (o + 16 <= end) __builtin_nontemporal_store(v[u], reinterpret_cast<u32x4 *>(dst + o));
                }
            }
        } else {
            const size_t eb = (size_t)p.elem_bytes;
            for (size_t o = begin + (size_t)tid * eb; o < end; o += (size_t)kDnThreads * eb) {
                if (eb == 4)
                    *reinterpret_cast<uint32_t *>(dst + o) = *reinterpret_cast<const uint32_t *>(src + o);
                else
                    *reinterpret_cast<uint16_t *>(dst + o) = *reinterpret_cast<const uint16_t *>(src + o);
            }
        }
    }

    auto copy_last_store = [&]() {
        if (copy_dst != nullptr) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const size_t o = copy_o0 + ((size_t)u * kDnThreads + tid) * 16;
                if (o + 16 <= copy_end) __builtin_nontemporal_store(copy_v[u], reinterpret_cast<u32x4 *>(copy_dst + o));
            }
            copy_dst = nullptr;
        }
    };

    f32x4 acc[CT][NT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[ct][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    // At most 16 channels (the paper's C_a): the contraction is split over the wavefronts by
    // input channel - wavefront w takes channels 4w .. 4w + 3, exactly the K of one
    // instruction, for ALL of the tile's runs of 16 pixels.  One A operand then serves 2 TH
    // independent accumulators (with one tile row per wavefront it served two, and a
    // compute unit with two blocks had four chains of dependent instructions per SIMD:
    // 42 % of the matrix rate), and nobody reads the same weights twice.  The four partial
    // results are added through LDS at the end.
    constexpr bool kSplitK = CT == 1;
    constexpr int NA = kSplitK ? 2 * TH : 1;
    f32x4 part[NA];
#pragma unroll
    for (int nt = 0; nt < NA; ++nt) part[nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    constexpr int kWPer = (kDenseMaxKs * CT * 256 + kDnThreads * 4 - 1) / (kDnThreads * 4);  // 16-byte pieces of a weight row per thread, at most
    for (int chunk = 0; chunk < CT; ++chunk) {
        // ---- the zero-extended halo tile of input channels 16*chunk .. +15 ----
        __syncthreads();  // the previous chunk's tile and weights are no longer read
        {
            const int hc = kDnTw + 2 * pad;
            const int total = 16 * HR * hc;
            constexpr int kFlight = 24;  // loads a thread has in flight: a round costs one trip to memory
            for (int i0 = 0; i0 < total; i0 += kFlight * kDnThreads) {
                float v[kFlight];
                unsigned inside = 0;  // bit u: element u lies in the image (the loads are unconditional, from clamped addresses)
#pragma unroll
                for (int u = 0; u < kFlight; ++u) {
                    const int idx = i0 + u * kDnThreads + tid;
                    const int ci = (int)dn_div((unsigned)idx, p.hp_mul, p.hp_shift), r2 = idx - ci * (HR * hc);
                    const int r = (int)dn_div((unsigned)r2, p.hc_mul, p.hc_shift), c = r2 - r * hc;
                    const int gy = y0 - pad + r, gx = x0 - pad + c, ch = 16 * chunk + ci;
                    const bool in = idx < total && ch < p.Ca && gy >= 0 && gy < H && gx >= 0 && gx < W;
                    v[u] = dn_load(xn + (in ? (size_t)ch * plane_px + (size_t)gy * W + gx : 0));
                    inside |= (in ? 1u : 0u) << u;
                }
                copy_last_store();
#pragma unroll
                for (int u = 0; u < kFlight; ++u) {
                    const int idx = i0 + u * kDnThreads + tid;
                    const int ci = (int)dn_div((unsigned)idx, p.hp_mul, p.hp_shift), r2 = idx - ci * (HR * hc);
                    const int r = (int)dn_div((unsigned)r2, p.hc_mul, p.hc_shift), c = r2 - r * hc;
                    if (idx < total) s_tile[ci * PLANE + r * PITCH + c] = ((inside >> u) & 1u) != 0 ? v[u] : 0.f;
                }
            }
        }
        // ---- kernel rows: row i's weights in LDS while row i + 1's are in flight in registers ----
        const float *wt_chunk = p.wt + (size_t)chunk * Ks * row_floats;
        const int pieces = row_floats / 4;  // 16-byte pieces per row
        f32x4 wreg[kWPer];
        auto fetch_row = [&](int i) {
#pragma unroll
            for (int u = 0; u < kWPer; ++u) {
                const int pc = u * kDnThreads + tid;
                wreg[u] = *reinterpret_cast<const f32x4 *>(wt_chunk + (size_t)i * row_floats + 4 * (pc < pieces ? pc : 0));
            }
        };
        fetch_row(0);
        for (int i = 0; i < Ks; ++i) {
            __syncthreads();  // row i - 1's taps are done with the weight area (and, for i == 0, the tile is written)
#pragma unroll
            for (int u = 0; u < kWPer; ++u) {
                const int pc = u * kDnThreads + tid;
                if (pc < pieces) *reinterpret_cast<f32x4 *>(s_w + 4 * pc) = wreg[u];
            }
            __syncthreads();
            if (i + 1 < Ks) fetch_row(i + 1);
            if constexpr (kSplitK) {
                // two operand sets take turns: tap j + 1's LDS reads are issued before tap j's
                // instructions (left to itself the compiler reads, waits and multiplies pair by pair)
                const float *wj = s_w + (4 * wave + kq) * 16 + l16;
                const float *tj = s_tile + (4 * wave + kq) * PLANE + i * PITCH + l16;
                auto fetch = [&](int j, float &a, float (&b)[NA]) {
                    a = wj[j * 256];
#pragma unroll
                    for (int nt = 0; nt < NA; ++nt) b[nt] = tj[(nt >> 1) * PITCH + 16 * (nt & 1) + j];
                };
                auto multiply = [&](float a, const float (&b)[NA]) {
#pragma unroll
                    for (int nt = 0; nt < NA; ++nt) part[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b[nt], part[nt], 0, 0, 0);
                };
                // (the reads are unconditional - beyond the last tap they repeat it - because behind
                // a branch the compiler no longer knows how many are in flight and waits for all)
                float a0, a1, b0[NA], b1[NA];
                fetch(0, a0, b0);
                for (int j = 0; j < Ks; j += 2) {
                    fetch(j + 1 < Ks ? j + 1 : Ks - 1, a1, b1);
                    __builtin_amdgcn_sched_barrier(0);
                    multiply(a0, b0);
                    __builtin_amdgcn_sched_barrier(0);
                    fetch(j + 2 < Ks ? j + 2 : Ks - 1, a0, b0);
                    __builtin_amdgcn_sched_barrier(0);
                    if (j + 1 < Ks) multiply(a1, b1);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            for (int j = 0; j < (kSplitK ? 0 : Ks); ++j) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    float b[NT];
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) {
                        const int r = RW * wave + (nt >> 1), c = 16 * (nt & 1);
                        b[nt] = s_tile[(4 * g + kq) * PLANE + (r + i) * PITCH + c + j + l16];
                    }
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct) {
                        const float a = s_w[((j * CT + ct) * 16 + 4 * g + kq) * 16 + l16];
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt)
                            acc[ct][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b[nt], acc[ct][nt], 0, 0, 0);
                    }
                }
            }
        }
        // ---- DK's nine depth-wise taps for the output channels of this chunk, from the same
        // tile: lane l holds output channels 16*chunk + 4*(l / 16) + r, r < 4, of pixel l % 16 ----
        if (p.dk != nullptr) {
            float d[4][9];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int co = 16 * chunk + 4 * kq + r;
#pragma unroll
                for (int k = 0; k < 9; ++k) d[r][k] = p.dk[((size_t)n * p.Ca + (co < p.Ca ? co : p.Ca - 1)) * 9 + k];
            }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int rr = RW * wave + (nt >> 1), c = 16 * (nt & 1);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float *src = s_tile + (4 * kq + r) * PLANE + (rr + pad - 1) * PITCH + c + pad - 1 + l16;
                    float s = 0.f;
#pragma unroll
                    for (int di = 0; di < 3; ++di)
#pragma unroll
                        for (int dj = 0; dj < 3; ++dj) s = fmaf(d[r][di * 3 + dj], src[di * PITCH + dj], s);
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct)  // (a constant index: the accumulators stay in registers)
                        if (ct == chunk) acc[ct][nt][r] += s;
                }
            }
        }
    }

    if constexpr (kSplitK) {
        // run nt of the tile belongs to wavefront nt / NT (as accumulator nt % NT); lane l's four
        // values of a run lie 16 bytes together, a wavefront's run 1 KiB, the four wavefronts'
        // copies of a run side by side
        constexpr int kPass = 8;  // runs per pass: 32 KiB of LDS
        f32x4 *s_red = reinterpret_cast<f32x4 *>(s_tile);
#pragma unroll
        for (int p0 = 0; p0 < NA; p0 += kPass) {
            __syncthreads();  // the tile (DK's taps) or the previous pass is no longer read
#pragma unroll
            for (int u = 0; u < kPass; ++u) s_red[((u * 4) + wave) * 64 + lane] = part[p0 + u];
            __syncthreads();
#pragma unroll
            for (int u = 0; u < kPass; ++u) {
                const int nt = p0 + u;
                if (nt / NT == wave) {  // wavefront-uniform
                    f32x4 sum = s_red[(u * 4 + 0) * 64 + lane];
#pragma unroll
                    for (int w = 1; w < 4; ++w) sum += s_red[(u * 4 + w) * 64 + lane];
#pragma unroll
                    for (int m = 0; m < NT; ++m)  // (a constant index: the accumulators stay in registers)
                        if (m == nt % NT) acc[0][m] += sum;
                }
            }
        }
    }

    // ---- store: one rounding to the storage type ----
    T *on = (T *)p.out + (size_t)n * p.C * plane_px;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int gy = y0 + RW * wave + (nt >> 1), gx = x0 + 16 * (nt & 1) + l16;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int co = 16 * ct + 4 * kq + r;
                if (co < p.Ca && gy < H && gx < W) dn_store(on + (size_t)co * plane_px + (size_t)gy * W + gx, acc[ct][nt][r]);
            }
        }
}

// ---------------------------------------------------------------------------------------
// Up to 16 channels: the contraction on v_mfma_f32_16x16x32_bf16.
//
// K of one instruction = two neighbouring taps of a kernel row x 16 input channels.  bf16
// storage: the stored values are the operands; each fp32 weight enters as two bf16 terms,
// w = hi + lo to 16 mantissa bits, so two instructions per operand pair, products exact,
// accumulation fp32.  fp32 storage (kernels up to 13 x 13): the bf16 instructions are sixteen
// times as fast as the fp32 ones, so every value and every weight is split exactly into three
// bf16 terms (dn_split3; one tile in LDS per term, three terms in the table) and the six
// products of terms whose orders add up to at most two are accumulated - what is left out
// lies below 2^-24 of a product, the size of fp32's own rounding.  The halo tile sits in LDS pixel-major, as cells of 16 bytes = eight
// channels of one pixel, in two half planes (channels 0-7, 8-15): the sixteen lanes that read
// one B operand's pixels read 256 consecutive bytes, the only pattern in which 16-byte LDS
// reads run at full rate.  The tile's columns start at x0 - 8, so that (W % 8 == 0, 16-byte
// aligned base) a thread fetches whole 16-byte pieces - eight pixels of each of eight
// channels - transposes them in registers and writes eight cells; the row pitch is odd in
// cells, lanes take consecutive rows, and the writes spread over all banks.
//
// The contraction is split over the four wavefronts by KERNEL ROW, every wavefront
// accumulating all runs of 16 pixels of the tile: for a pair of tap columns a wavefront
// holds the A operands of its block of 3-5 neighbouring kernel rows and walks down the tile
// rows once - a B operand (tile row R, half h) serves every kernel row i of the block with
// an output row R - i in the tile, so one 1 KiB read feeds up to 2 x 5 instructions instead
// of two (read once per tap pair and run, the same loop was bound by the LDS as much as by
// the matrix cores).  Which wavefront takes the larger block rotates with the pair, so that
// the four end together; the next pair's A operands (from the rearranged table in memory)
// travel during the walk.  The four partial results meet in LDS as in the fp32 kernel.  An
// odd kernel leaves the last pair's second column empty: those lanes read the first
// column's pixels again, against zero weights.
// ---------------------------------------------------------------------------------------
constexpr int kBfCols = 48;   // cells per tile row: columns x0 - 8 .. x0 + 39, six aligned pieces of eight
constexpr int kBfPitch = 49;  // row pitch in cells

// cells in one half plane of the tile; first cell behind the tile and behind the 32 KiB (2048
// cells) that the partial results pass through; the block's LDS bytes (DK sits at the end)
__host__ __device__ constexpr int bf_half_cells(int Kse, int th) { return (th + Kse - 1) * kBfPitch; }
__host__ __device__ constexpr int bf_aux_cell(int Kse, int th, int nx)
{
    return nx * 2 * bf_half_cells(Kse, th) < 2048 ? 2048 : nx * 2 * bf_half_cells(Kse, th);
}
inline size_t bf_lds_bytes(int Kse, int th, int nx) { return (size_t)bf_aux_cell(Kse, th, nx) * 16 + 16 * 9 * sizeof(float); }

__device__ __forceinline__ void dn_split3(float v, uint16_t (&t)[3]) { dw_split3(v, t); }

// the A-operand table (dense_table_entry), one thread per entry
__global__ void dense_weights_bf16_kernel(const float *lk, int Ca, int Ks, int Kse, int nw, uint32_t *wa)
{
    const int idx = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (idx < dense_table_entries(Kse)) dense_table_entry(lk, Ca, Ks, Kse, nw, wa, idx);
}

template <typename T, int KS, int TH>
__global__ __launch_bounds__(kDnThreads, 2) void dense_bf16_kernel(const DenseParams p)
{
    typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    constexpr bool kF32 = std::is_same<T, float>::value;
    constexpr int NX = kF32 ? 3 : 1;  // bf16 terms of a stored value (one tile in LDS per term)
    constexpr int NW = kF32 ? 3 : 2;  // bf16 terms of a weight
    constexpr int NA = 2 * TH;  // runs of 16 pixels in the tile: run nt = row nt / 2, columns 16 (nt % 2) ..
    constexpr int NT = TH / 2;  // runs whose results a wavefront ends up with
    constexpr int pad = (KS - 1) / 2, HR = TH + 2 * pad, HP = HR * kBfPitch;
    const int tid = (int)threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, kq = lane >> 4;
    const int H = p.H, W = p.W;
    char *s_bytes = reinterpret_cast<char *>(dn_lds);
    u32x4 *s_cells = reinterpret_cast<u32x4 *>(dn_lds);  // [NX terms][2 halves][HR][kBfPitch] cells
    constexpr int TILE = 2 * HP;                          // cells of one term's tile
    float *s_dk = reinterpret_cast<float *>(s_cells + bf_aux_cell(KS, TH, NX));
    const size_t plane_px = (size_t)H * W;

    // Blocks go to the chip's eight dies round robin; each die gets a contiguous eighth of the
    // tiles, so that neighbouring tiles (shared halos) meet in one L2.
    const unsigned nblk = gridDim.x, die = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
    const unsigned qd = nblk / kXcds, rem = nblk % kXcds;
    const unsigned tile_id = die * qd + (die < rem ? die : rem) + slot;
    const unsigned per_img = (unsigned)(p.tiles_x * p.tiles_y);
    const unsigned n = tile_id / per_img, t_in = tile_id - n * per_img;
    const int tyi = (int)(t_in / (unsigned)p.tiles_x), txi = (int)(t_in - (unsigned)tyi * p.tiles_x);
    const int y0 = tyi * TH, x0 = txi * kDnTw;
    const T *xn = (const T *)p.x + (size_t)n * p.C * plane_px;

    // ---- the block's share of the pass-through copy (Eq. 4 lines 1 and 4): up to three rounds
    // of 16 KiB are asked for at once, in front of the tile, and stored behind the tile's loads
    // (copy_last_store): one trip to memory for both, while no other registers are live ----
    constexpr int kCopyRounds = 3;
    constexpr int kWalkGrains = 2;  // 16-byte accesses per thread and walk of the contraction
    constexpr size_t kWalkCopy = (size_t)((KS + 1) / 2) * kWalkGrains * kDnThreads * 16;
    const char *walk_src = reinterpret_cast<const char *>(p.wt);  // (a readable, aligned address for the clamped loads of a walk with nothing to copy)
    char *walk_dst = nullptr;
    size_t walk_len = 0;
    u32x4 copy_v[4 * kCopyRounds] = {};
    size_t copy_o0 = 0, copy_end = 0;
    char *copy_dst = nullptr;
    if (p.idt_len > 0) {
        const char *src = (const char *)p.x + (size_t)n * p.img_bytes + p.idt_off;
        char *dst = (char *)p.out + (size_t)n * p.img_bytes + p.idt_off;
        const size_t begin0 = (size_t)t_in * p.copy_share < p.idt_len ? (size_t)t_in * p.copy_share : p.idt_len;
        const size_t end = begin0 + p.copy_share < p.idt_len ? begin0 + p.copy_share : p.idt_len;
        // (with vector accesses, the first kWalkCopy bytes of the share travel during the contraction, see there)
        const size_t begin = p.copy_vec ? (begin0 + kWalkCopy < end ? begin0 + kWalkCopy : end) : begin0;
        if (p.copy_vec && begin > begin0) walk_src = src + begin0, walk_dst = dst + begin0, walk_len = begin - begin0;
        if (p.copy_vec) {
            constexpr size_t kGroup = (size_t)4 * kCopyRounds * kDnThreads * 16;
            for (size_t o0 = begin; o0 < end; o0 += kGroup) {
                u32x4 v[4 * kCopyRounds];
#pragma unroll
                for (int u = 0; u < 4 * kCopyRounds; ++u) {
                    const size_t o = o0 + ((size_t)u * kDnThreads + tid) * 16;
                    v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + (o + 16 <= end ? o : begin)));
                }
                if (o0 + kGroup >= end) {  // the last group (block-uniform)
#pragma unroll
                    for (int u = 0; u < 4 * kCopyRounds; ++u) copy_v[u] = v[u];
                    copy_o0 = o0, copy_end = end, copy_dst = dst;
                    break;
                }
#pragma unroll
                for (int u = 0; u < 4 * kCopyRounds; ++u) {
                    const size_t o = o0 + ((size_t)u * kDnThreads + tid) * 16;
                    if (o + 16 <= end) __builtin_nontemporal_store(v[u], reinterpret_cast<u32x4 *>(dst + o));
                }
            }
        } else {
            typedef typename std::conditional<kF32, uint32_t, uint16_t>::type E;
            for (size_t o = begin + (size_t)tid * sizeof(E); o < end; o += (size_t)kDnThreads * sizeof(E))
                *reinterpret_cast<E *>(dst + o) = *reinterpret_cast<const E *>(src + o);
        }
    }
    auto copy_last_store = [&]() {
        if (copy_dst != nullptr) {
#pragma unroll
            for (int u = 0; u < 4 * kCopyRounds; ++u) {
                const size_t o = copy_o0 + ((size_t)u * kDnThreads + tid) * 16;
                if (o + 16 <= copy_end) __builtin_nontemporal_store(copy_v[u], reinterpret_cast<u32x4 *>(copy_dst + o));
            }
            copy_dst = nullptr;
        }
    };

    // DK of this image goes to LDS beside the tile (asked for now, read after the contraction)
    float dk_v = 0.f;
    if (p.dk != nullptr && tid < 16 * 9) dk_v = p.dk[(size_t)n * p.Ca * 9 + (tid < p.Ca * 9 ? tid : 0)];

    // ---- the zero-extended halo tile, pixel-major ----
    if (kF32 && p.fill_vec) {
        // fp32 storage: the same tasks, 32 bytes (eight pixels) of each of eight channels per task,
        // every value split into its three terms on the way to the three tiles
        if constexpr (kF32) {
            constexpr int tasks = 2 * (kBfCols / 8) * HR, KT = (tasks + kDnThreads - 1) / kDnThreads;
            u32x4 v[KT][8][2];
            bool in[KT];
#pragma unroll
            for (int k = 0; k < KT; ++k) {
                const int task = k * kDnThreads + tid;
                const int r = task % HR, rest = task / HR, pc = rest % (kBfCols / 8), h2 = rest / (kBfCols / 8);
                const int gy = y0 - pad + r, gx = x0 - 8 + 8 * pc;
                in[k] = task < tasks && gy >= 0 && gy < H && gx >= 0 && gx < W;
                const size_t o = in[k] ? (size_t)gy * W + gx : 0;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int ch = 8 * h2 + e;
                    const float *src = xn + (ch < p.Ca ? (size_t)ch * plane_px : 0) + o;
                    v[k][e][0] = *reinterpret_cast<const u32x4 *>(src);
                    v[k][e][1] = *reinterpret_cast<const u32x4 *>(src + 4);
                }
            }
            copy_last_store();
#pragma unroll
            for (int k = 0; k < KT; ++k) {
                const int task = k * kDnThreads + tid;
                const int r = task % HR, rest = task / HR, pc = rest % (kBfCols / 8), h2 = rest / (kBfCols / 8);
                u32x4 *dst = s_cells + h2 * HP + r * kBfPitch + 8 * pc;
#pragma unroll
                for (int d = 0; d < 8; ++d) {
                    u32x4 cell[3];  // pixel d of the piece, one cell per term
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        uint16_t ta[3], tb[3];
                        const bool a_in = in[k] && 8 * h2 + 2 * w < p.Ca, b_in = in[k] && 8 * h2 + 2 * w + 1 < p.Ca;
                        dn_split3(a_in ? __uint_as_float(v[k][2 * w][d >> 2][d & 3]) : 0.f, ta);
                        dn_split3(b_in ? __uint_as_float(v[k][2 * w + 1][d >> 2][d & 3]) : 0.f, tb);
#pragma unroll
                        for (int t = 0; t < 3; ++t) cell[t][w] = (uint32_t)ta[t] | ((uint32_t)tb[t] << 16);
                    }
                    if (task < tasks) {
#pragma unroll
                        for (int t = 0; t < 3; ++t) dst[t * TILE + d] = cell[t];
                    }
                }
            }
        }
    } else if (p.fill_vec) {
        // task = (half, piece of eight columns, row), lanes on consecutive rows; at most two per thread
        constexpr int tasks = 2 * (kBfCols / 8) * HR;
        u32x4 v[2][8];
        bool in[2];
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int task = k * kDnThreads + tid;
            const int r = task % HR, rest = task / HR, pc = rest % (kBfCols / 8), h2 = rest / (kBfCols / 8);
            const int gy = y0 - pad + r, gx = x0 - 8 + 8 * pc;
            in[k] = task < tasks && gy >= 0 && gy < H && gx >= 0 && gx < W;
            const size_t o = in[k] ? (size_t)gy * W + gx : 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int ch = 8 * h2 + e;
                v[k][e] = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const bf16d *>(p.x) + (size_t)n * p.C * plane_px +
                                                           (ch < p.Ca ? (size_t)ch * plane_px : 0) + o);
            }
        }
        copy_last_store();
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int task = k * kDnThreads + tid;
            const int r = task % HR, rest = task / HR, pc = rest % (kBfCols / 8), h2 = rest / (kBfCols / 8);
            u32x4 *dst = s_cells + h2 * HP + r * kBfPitch + 8 * pc;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                u32x4 c0, c1;  // the cells of pixels 2 d and 2 d + 1
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const bool a_in = in[k] && 8 * h2 + 2 * w < p.Ca, b_in = in[k] && 8 * h2 + 2 * w + 1 < p.Ca;
                    const uint32_t a = a_in ? v[k][2 * w][d] : 0u, b = b_in ? v[k][2 * w + 1][d] : 0u;
                    c0[w] = (a & 0xffffu) | (b << 16);
                    c1[w] = (a >> 16) | (b & 0xffff0000u);
                }
                if (task < tasks) {
                    dst[2 * d] = c0;
                    dst[2 * d + 1] = c1;
                }
            }
        }
    } else {
        // any width and alignment: element by element
        copy_last_store();
        constexpr int total = 16 * HR * kBfCols;
        for (int i0 = 0; i0 < total; i0 += 8 * kDnThreads) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = i0 + u * kDnThreads + tid;
                const int ci = idx / (HR * kBfCols), r2 = idx - ci * (HR * kBfCols), r = r2 / kBfCols, c = r2 - r * kBfCols;
                const int gy = y0 - pad + r, gx = x0 - 8 + c;
                const bool ok = idx < total && ci < p.Ca && gy >= 0 && gy < H && gx >= 0 && gx < W;
                const float raw = dn_load(xn + (ok ? (size_t)ci * plane_px + (size_t)gy * W + gx : 0));
                v[u] = ok ? raw : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = i0 + u * kDnThreads + tid;
                const int ci = idx / (HR * kBfCols), r2 = idx - ci * (HR * kBfCols), r = r2 / kBfCols, c = r2 - r * kBfCols;
                uint16_t t3[3];
                dn_split3(v[u], t3);  // (bf16 storage: the value is its own first term)
                if (idx < total) {
#pragma unroll
                    for (int t = 0; t < NX; ++t)
                        *reinterpret_cast<uint16_t *>(s_bytes + (size_t)(t * TILE + (ci >> 3) * HP + r * kBfPitch + c) * 16 + (ci & 7) * 2) = t3[t];
                }
            }
        }
    }
    if (tid < 16 * 9) s_dk[tid] = dk_v;
    __syncthreads();

    // ---- the contraction ----
    f32x4 part[NA];
#pragma unroll
    for (int nt = 0; nt < NA; ++nt) part[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    {
        constexpr int NJP = (KS + 1) / 2;                // pairs of tap columns
        constexpr int kBase = KS / 4, kExtra = KS % 4;   // kernel rows per wavefront: kBase, one more for kExtra of the four
        constexpr int MB = kBase + 1;                    // (KS is odd: kExtra > 0)
        constexpr int NR = TH + MB - 1;                  // tile rows a block of MB kernel rows walks
        const u32x4 *wa = reinterpret_cast<const u32x4 *>(p.wt) + lane;
        // this wavefront's block of kernel rows for pair jp: rows i0 .. i0 + cnt - 1
        auto rows_of = [&](int jp, int &i0, int &cnt) {
            const int pos = (wave - jp) & 3;
            i0 = pos * kBase + (pos < kExtra ? pos : kExtra);
            cnt = kBase + (pos < kExtra ? 1 : 0);
        };
        auto fetch_a = [&](int jp, u32x4 (&a)[MB][NW]) {
            int i0, cnt;
            rows_of(jp, i0, cnt);
#pragma unroll
            for (int m = 0; m < MB; ++m) {
                int i = i0 + (m < cnt ? m : 0);
                i = i < KS ? i : KS - 1;
#pragma unroll
                for (int t = 0; t < NW; ++t) a[m][t] = wa[((size_t)(jp * KS + i) * NW + t) * 64];
            }
        };
        // the products of a value's and a weight's terms that are accumulated, small ones first:
        // bf16 storage (value, lo) and (value, hi); fp32 storage the six products of terms whose
        // orders add up to at most two - the three left out lie below 2^-24 of the product
        constexpr int NP = kF32 ? 6 : 2;
        constexpr int kPx[6] = {2, 0, 1, 1, 0, 0}, kPw[6] = {0, 2, 1, 0, 1, 0};
        auto px = [&](int q) { return kF32 ? kPx[q] : 0; };
        auto pw = [&](int q) { return kF32 ? kPw[q] : 1 - q; };
        auto mma = [&](const u32x4 &a, const u32x4 &b, f32x4 &c) {
            c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
        };
        // a walk's piece of the pass-through copy: asked for at its start, behind the next
        // pair's A operands (which are waited for first), stored at the end of the NEXT walk -
        // a trip to memory takes longer than one walk
        auto copy_ask = [&](int jp, u32x4 (&cv)[kWalkGrains]) {
#pragma unroll
            for (int g = 0; g < kWalkGrains; ++g) {
                const size_t o = (((size_t)jp * kWalkGrains + g) * kDnThreads + tid) * 16;
                cv[g] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(walk_src + (o + 16 <= walk_len ? o : 0)));
            }
        };
        auto copy_put = [&](int jp, const u32x4 (&cv)[kWalkGrains]) {
#pragma unroll
            for (int g = 0; g < kWalkGrains; ++g) {
                const size_t o = (((size_t)jp * kWalkGrains + g) * kDnThreads + tid) * 16;
                if (jp >= 0 && o + 16 <= walk_len) __builtin_nontemporal_store(cv[g], reinterpret_cast<u32x4 *>(walk_dst + o));
            }
        };
        auto walk = [&](int jp, const u32x4 (&a)[MB][NW], u32x4 (&a_next)[MB][NW], u32x4 (&cv)[kWalkGrains],
                        const u32x4 (&cv_before)[kWalkGrains]) {
            int i0, cnt;
            rows_of(jp, i0, cnt);
            fetch_a(jp + 1 < NJP ? jp + 1 : jp, a_next);
            copy_ask(jp, cv);
            const bool full = cnt == MB;  // wavefront-uniform
            // this lane's B operand for tile row i0, half 0: its tap column's shift (the empty
            // column reads the one before it), its half plane, its pixel
            int j = 2 * jp + (kq >> 1);
            j = j < KS ? j : KS - 1;
            const char *bp = s_bytes + (size_t)((kq & 1) * HP + i0 * kBfPitch + j + 8 - pad + l16) * 16;
            u32x4 b[2][2][NX];
            auto read_b = [&](int R, u32x4 (&bb)[2][NX]) {
#pragma unroll
                for (int t = 0; t < NX; ++t) {
                    bb[0][t] = *reinterpret_cast<const u32x4 *>(bp + (t * TILE + R * kBfPitch) * 16);
                    bb[1][t] = *reinterpret_cast<const u32x4 *>(bp + (t * TILE + R * kBfPitch) * 16 + 256);
                }
            };
            read_b(0, b[0]);
#pragma unroll
            for (int R = 0; R < NR; ++R) {
                // tile row R + 1 (the last one serves the block's last kernel row only)
                if (R + 1 < NR - 1) read_b(R + 1, b[(R + 1) & 1]);
                if (R + 1 == NR - 1 && full) read_b(R + 1, b[(R + 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = 0; q < NP; ++q)
#pragma unroll
                    for (int m = 0; m < MB - 1; ++m)
                        if (R - m >= 0 && R - m < TH) {
                            mma(a[m][pw(q)], b[R & 1][0][px(q)], part[2 * (R - m)]);
                            mma(a[m][pw(q)], b[R & 1][1][px(q)], part[2 * (R - m) + 1]);
                        }
                if (R - (MB - 1) >= 0 && R - (MB - 1) < TH && full) {
#pragma unroll
                    for (int q = 0; q < NP; ++q) {
                        mma(a[MB - 1][pw(q)], b[R & 1][0][px(q)], part[2 * (R - (MB - 1))]);
                        mma(a[MB - 1][pw(q)], b[R & 1][1][px(q)], part[2 * (R - (MB - 1)) + 1]);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            copy_put(jp - 1, cv_before);
        };
        u32x4 a0[MB][NW], a1[MB][NW], cv0[kWalkGrains] = {}, cv1[kWalkGrains] = {};
        fetch_a(0, a0);
#pragma unroll
        for (int jp = 0; jp < NJP; jp += 2) {
            walk(jp, a0, a1, cv0, cv1);
            if (jp + 1 < NJP) walk(jp + 1, a1, a0, cv1, cv0);
        }
        copy_put(NJP - 1, (NJP - 1) % 2 == 0 ? cv0 : cv1);
    }

    // ---- DK's nine depth-wise taps for the runs this wavefront ends up with, from the same
    // tile: lane l holds output channels 4 (l / 16) + r, r < 4, of pixel l % 16 ----
    f32x4 acc[NT];
#pragma unroll
    for (int m = 0; m < NT; ++m) acc[m] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (p.dk != nullptr) {
        float d[4][9];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int k = 0; k < 9; ++k) d[r][k] = s_dk[(4 * kq + r) * 9 + k];
#pragma unroll
        for (int m = 0; m < NT; ++m) {
            const int nt = wave * NT + m, rr = nt >> 1, c = 16 * (nt & 1);
            const char *src = s_bytes + (size_t)((kq >> 1) * HP + (rr + pad - 1) * kBfPitch + c + l16 + 7) * 16 + 8 * (kq & 1);
#pragma unroll
            for (int di = 0; di < 3; ++di)
#pragma unroll
                for (int dj = 0; dj < 3; ++dj) {
                    float xv[4] = {0.f, 0.f, 0.f, 0.f};  // the stored value: the sum of its terms, smallest first (exact)
#pragma unroll
                    for (int t = NX - 1; t >= 0; --t) {
                        const u32x2 v = *reinterpret_cast<const u32x2 *>(src + (t * TILE + di * kBfPitch + dj) * 16);
                        xv[0] += __uint_as_float(v[0] << 16);
                        xv[1] += __uint_as_float(v[0] & 0xffff0000u);
                        xv[2] += __uint_as_float(v[1] << 16);
                        xv[3] += __uint_as_float(v[1] & 0xffff0000u);
                    }
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[m][r] = fmaf(d[r][di * 3 + dj], xv[r], acc[m][r]);
                }
        }
    }

    // ---- the four wavefronts' partial results: run nt goes to wavefront nt / NT ----
    {
        constexpr int kPass = NA < 8 ? NA : 8;  // runs per pass: 32 KiB of LDS
        f32x4 *s_red = reinterpret_cast<f32x4 *>(dn_lds);
#pragma unroll
        for (int p0 = 0; p0 < NA; p0 += kPass) {
            __syncthreads();  // the tile (DK's taps) or the previous pass is no longer read
#pragma unroll
            for (int u = 0; u < kPass; ++u) s_red[((u * 4) + wave) * 64 + lane] = part[p0 + u];
            __syncthreads();
#pragma unroll
            for (int u = 0; u < kPass; ++u) {
                const int nt = p0 + u;
                if (nt / NT == wave) {  // wavefront-uniform
                    f32x4 sum = s_red[(u * 4 + 0) * 64 + lane];
#pragma unroll
                    for (int w = 1; w < 4; ++w) sum += s_red[(u * 4 + w) * 64 + lane];
#pragma unroll
                    for (int m = 0; m < NT; ++m)  // (a constant index: the accumulators stay in registers)
                        if (m == nt % NT) acc[m] += sum;
                }
            }
        }
    }

    // ---- store: one rounding to the storage type ----
    T *on = (T *)p.out + (size_t)n * p.C * plane_px;
#pragma unroll
    for (int m = 0; m < NT; ++m) {
        const int nt = wave * NT + m;
        const int gy = y0 + (nt >> 1), gx = x0 + 16 * (nt & 1) + l16;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int co = 4 * kq + r;
            if (co < p.Ca && gy < H && gx < W) dn_store(on + (size_t)co * plane_px + (size_t)gy * W + gx, acc[m][r]);
        }
    }
}

template <typename T, int KS, int TH>
hipError_t launch_bf16_kt(const DenseParams &p, unsigned grid, hipStream_t s)
{
    const size_t lds = bf_lds_bytes(KS, TH, std::is_same<T, float>::value ? 3 : 1);
    static bool granted = false;
    if (lds > 48 * 1024 && !granted) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&dense_bf16_kernel<T, KS, TH>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        granted = true;
    }
    hipLaunchKernelGGL((dense_bf16_kernel<T, KS, TH>), dim3(grid), dim3(kDnThreads), lds, s, p);
    return hipGetLastError();
}

template <typename T, int TH>
hipError_t launch_bf16(const DenseParams &p, unsigned grid, hipStream_t s)
{
    switch (p.Ks) {
    case 3: return launch_bf16_kt<T, 3, TH>(p, grid, s);
    case 5: return launch_bf16_kt<T, 5, TH>(p, grid, s);
    case 7: return launch_bf16_kt<T, 7, TH>(p, grid, s);
    case 9: return launch_bf16_kt<T, 9, TH>(p, grid, s);
    case 11: return launch_bf16_kt<T, 11, TH>(p, grid, s);
    case 13: return launch_bf16_kt<T, 13, TH>(p, grid, s);
    }
    if constexpr (!std::is_same<T, float>::value) {  // (fp32 storage: three tiles in LDS, kernels up to 13 x 13)
        if (p.Ks == 15) return launch_bf16_kt<T, 15, TH>(p, grid, s);
        if (p.Ks == 17) return launch_bf16_kt<T, 17, TH>(p, grid, s);
    }
    return hipErrorInvalidValue;
}

template <typename T, int CT, int TH>
hipError_t launch_ct(const DenseParams &p, unsigned grid, size_t lds, hipStream_t s)
{
    static size_t granted = 48 * 1024;
    if (lds > granted) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&dense_kernel<T, CT, TH>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        granted = lds;
    }
    hipLaunchKernelGGL((dense_kernel<T, CT, TH>), dim3(grid), dim3(kDnThreads), lds, s, p);
    return hipGetLastError();
}

template <typename T, int TH>
hipError_t launch_t(const DenseParams &p, int ct, unsigned grid, size_t lds, hipStream_t s)
{
    switch (ct) {
    case 1: return launch_ct<T, 1, TH>(p, grid, lds, s);
    case 2: return launch_ct<T, 2, TH>(p, grid, lds, s);
    case 3: return launch_ct<T, 3, TH>(p, grid, lds, s);
    case 4: return launch_ct<T, 4, TH>(p, grid, lds, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace

__attribute__((visibility("hidden"))) hipError_t launch_dense_weights(const float *lk, int Ca, int Ks, bool bf16, float *wt, hipStream_t s)
{
    const int Kse = dense_effective_ks(Ks);
    if (dense_on_bf16_mfma(Ca, Ks, bf16)) {
        const int threads = dense_table_entries(Kse);
        hipLaunchKernelGGL(dense_weights_bf16_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, lk, Ca, Ks, Kse,
                           bf16 ? 2 : 3, reinterpret_cast<uint32_t *>(wt));
        return hipGetLastError();
    }
    const size_t total = dense_weight_floats(Ca, Ks);
    if (total == 0) return hipSuccess;
    hipLaunchKernelGGL(dense_weights_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, lk, Ca, Ks, Kse, wt, total);
    return hipGetLastError();
}

__attribute__((visibility("hidden"))) hipError_t launch_dense(const DenseParams &p_in, bool bf16, hipStream_t s)
{
    DenseParams p = p_in;
    p.Ks = dense_effective_ks(p.Ks);  // the kernel walks the embedding kernel (launch_dense_weights)
    if (p.Ca < 1 || p.Ca > kDenseMaxCa || p.Ks < 1 || p.Ks > kDenseMaxKs) return hipErrorInvalidValue;
    const int ct = (p.Ca + 15) / 16;
    // 8-row tiles, or 4-row ones while those are needed to give every compute unit two blocks
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return hipErrorInvalidDevice;
        cus = n > 0 ? n : 1;
    }
    p.tiles_x = (p.W + kDnTw - 1) / kDnTw;
    const size_t blocks8 = (size_t)p.tiles_x * ((p.H + 7) / 8) * p.N;
    const bool matrix_bf16 = dense_on_bf16_mfma(p.Ca, p.Ks, bf16);
    // (fp32 storage on the bf16 instructions keeps three tiles in LDS: 4-row tiles, two blocks per compute unit)
    const int th = (blocks8 >= 2 * (size_t)cus && !(matrix_bf16 && !bf16)) ? 8 : 4;
    p.tiles_y = (p.H + th - 1) / th;
    const size_t per_img = (size_t)p.tiles_x * p.tiles_y;
    const size_t grid = per_img * p.N;
    if (grid >= ((size_t)1 << 31)) return hipErrorInvalidValue;
    if (p.idt_len > 0) {
        // every block of an image moves an equal share, in whole 16 KiB rounds when vector accesses apply
        const size_t grain = p.copy_vec ? (size_t)4 * kDnThreads * 16 : (size_t)p.elem_bytes;
        size_t share = (p.idt_len + per_img - 1) / per_img;
        share = (share + grain - 1) / grain * grain;
        p.copy_share = share;
    }
    if (matrix_bf16) {
        p.fill_vec = (p.W % 8 == 0) && ((uintptr_t)p.x % 16 == 0);
        if (!bf16) return launch_bf16<float, 4>(p, (unsigned)grid, s);
        return th == 8 ? launch_bf16<bf16d, 8>(p, (unsigned)grid, s) : launch_bf16<bf16d, 4>(p, (unsigned)grid, s);
    }
    int hr, pitch, plane;
    dense_geom(p.Ks, th, hr, pitch, plane);
    const unsigned hc = (unsigned)(kDnTw + 2 * ((p.Ks - 1) / 2));
    dn_make_div(hc, p.hc_mul, p.hc_shift);
    dn_make_div((unsigned)hr * hc, p.hp_mul, p.hp_shift);
    size_t lds = ((size_t)16 * plane + (size_t)p.Ks * ct * 256) * sizeof(float);
    // (up to 16 channels: the wavefronts' partial results pass through the same LDS, 32 KiB at a time)
    if (ct == 1 && lds < (size_t)8 * 4 * 64 * 16) lds = (size_t)8 * 4 * 64 * 16;
    if (th == 8)
        return bf16 ? launch_t<bf16d, 8>(p, ct, (unsigned)grid, lds, s) : launch_t<float, 8>(p, ct, (unsigned)grid, lds, s);
    return bf16 ? launch_t<bf16d, 4>(p, ct, (unsigned)grid, lds, s) : launch_t<float, 4>(p, ct, (unsigned)grid, lds, s);
}

}  // namespace esc

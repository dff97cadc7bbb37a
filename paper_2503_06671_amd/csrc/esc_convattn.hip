// ConvAttn forward for gfx950 (MI355X): hand-written HIP kernels and the C ABI
// declared in include/esc_convattn.h.
//
// The operation is Eq. 4 of the ESC paper with the depth-wise large kernel of
// the paragraph around Eq. 5.  Four kernel families, all plain fp32 vector
// arithmetic (a depth-wise convolution has no reduction shared between outputs,
// so there is nothing to feed a matrix core with):
//
//   pool_kernel   GAP partial sums of the attention slice, one fixed-size slab
//                 per block, fixed reduction order (bit-reproducible)
//   gen_kernel    per image: finish the GAP, run the kernel estimator, write DK
//   conv_kernel   fused LK + DK depth-wise convolution from one LDS halo tile,
//                 4 x RY outputs per thread in registers
//   copy_kernel   pass-through of the identity channels
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "esc_convattn.h"

namespace {

constexpr int kThreads = 256;      // every kernel uses 4 wavefronts per block
constexpr int kTileW = 64;         // conv tile width: 16 lanes x 4 outputs
constexpr int kPoolSlab = 4096;    // elements per GAP partial sum
constexpr int kMaxCa = 256;
constexpr int kMaxHidden = 256;
constexpr int kMaxKs = 31;
constexpr size_t kWsAlign = 256;

struct bf16_t {
    uint16_t bits;
};
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return __uint_as_float((uint32_t)v.bits << 16); }

// fp32 -> bf16, round to nearest even, NaN kept quiet
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ void store1(float *p, float v) { *p = v; }
__device__ __forceinline__ void store1(bf16_t *p, float v) { p->bits = f32_to_bf16_bits(v); }

__device__ __forceinline__ void store4(float *p, const float *v)
{
    *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void store4(bf16_t *p, const float *v)
{
    uint2 w;
    w.x = (uint32_t)f32_to_bf16_bits(v[0]) | ((uint32_t)f32_to_bf16_bits(v[1]) << 16);
    w.y = (uint32_t)f32_to_bf16_bits(v[2]) | ((uint32_t)f32_to_bf16_bits(v[3]) << 16);
    *reinterpret_cast<uint2 *>(p) = w;
}

// ---------------------------------------------------------------------------
// GAP partial sums (Eq. 4 line 2, first half).  Block b owns slab b % nslab of
// plane b / nslab.  The decomposition depends on H*W only, and every sum runs in
// a fixed order, so a batch gives bit-identical results to its images run alone.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void pool_kernel(const T *__restrict__ x,
                                                        float *__restrict__ partials, int C, int Ca,
                                                        int HW, int nslab)
{
    __shared__ float wsum[kThreads / 64];
    const int slab = blockIdx.x % nslab;
    const int nc = blockIdx.x / nslab;
    const int n = nc / Ca, c = nc % Ca;
    const T *plane = x + ((size_t)n * C + c) * (size_t)HW;
    const int base = slab * kPoolSlab;
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < kPoolSlab / kThreads; ++k) {
        int idx = base + k * kThreads + (int)threadIdx.x;
        if (idx < HW) s += to_f32(plane[idx]);
    }
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = wsum[0];
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) t += wsum[w];
        partials[(size_t)nc * nslab + slab] = t;
    }
}

// ---------------------------------------------------------------------------
// Kernel estimator (Eq. 4 line 2, second half).  One block per image.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float gelu_erf(float v) { return 0.5f * v * (1.f + erff(v * 0.70710678118654752440f)); }

__global__ __launch_bounds__(kThreads) void gen_kernel(const float *__restrict__ partials, int nslab,
                                                       float hw, int Ca, int hidden,
                                                       const float *__restrict__ w_down,
                                                       const float *__restrict__ b_down,
                                                       const float *__restrict__ w_up,
                                                       const float *__restrict__ b_up,
                                                       float *__restrict__ dk)
{
    __shared__ float g[kMaxCa];
    __shared__ float t[kMaxHidden];
    const int n = blockIdx.x;
    for (int c = threadIdx.x; c < Ca; c += kThreads) {
        const float *p = partials + ((size_t)n * Ca + c) * nslab;
        float s = 0.f;
        for (int k = 0; k < nslab; ++k) s += p[k];
        g[c] = s / hw;
    }
    __syncthreads();
    const float *in = g;
    int K = Ca;
    if (hidden > 0) {
        for (int m = threadIdx.x; m < hidden; m += kThreads) {
            float s = b_down ? b_down[m] : 0.f;
            for (int k = 0; k < Ca; ++k) s = fmaf(w_down[(size_t)m * Ca + k], g[k], s);
            t[m] = gelu_erf(s);
        }
        __syncthreads();
        in = t;
        K = hidden;
    }
    for (int o = threadIdx.x; o < 9 * Ca; o += kThreads) {
        float s = b_up ? b_up[o] : 0.f;
        for (int k = 0; k < K; ++k) s = fmaf(w_up[(size_t)o * K + k], in[k], s);
        dk[(size_t)n * 9 * Ca + o] = s;
    }
}

// ---------------------------------------------------------------------------
// Fused depth-wise convolution (Eq. 4 line 3).  A block owns a 64 x (16*RY)
// output tile of one (image, channel) plane.  The zero-extended halo tile sits in
// LDS as fp32; thread (tx, ty) produces outputs x = 4*tx..4*tx+3 of rows
// ty*RY..ty*RY+RY-1.  Each LDS row segment it loads (KS+3 values, 16-byte reads)
// feeds up to RY kernel rows, and the kernel weights are wave-uniform, so the tap
// loop is FMA with a scalar-register multiplier.  DK's nine taps run afterwards
// from the same tile.
// ---------------------------------------------------------------------------
template <int KS, int RY, typename T>
__global__ __launch_bounds__(kThreads) void conv_kernel(const T *__restrict__ x, T *__restrict__ out,
                                                        const float *__restrict__ lk, long lk_cstride,
                                                        const float *__restrict__ dk, int C, int Ca,
                                                        int H, int W, int tiles_x, int tiles_y,
                                                        int vec_ok)
{
    constexpr int P = (KS - 1) / 2;
    constexpr int PH = P > 1 ? P : 1;  // halo width: DK's 3x3 needs one pixel even when Ks == 1
    constexpr int OFF = PH - P;        // where the LK window starts inside the halo
    constexpr int TH = 16 * RY;
    constexpr int HR = TH + 2 * PH;
    constexpr int HC = kTileW + 2 * PH;
    constexpr int PITCH = (HC + 3) & ~3;
    constexpr int NV = (KS + 3 + 3) & ~3;  // values a thread reads per tile row
    constexpr bool kUnrollRows = (KS <= 13);
    __shared__ __align__(16) float tile[HR * PITCH];

    int b = blockIdx.x;
    const int txi = b % tiles_x;
    b /= tiles_x;
    const int tyi = b % tiles_y;
    const int nc = b / tiles_y;
    const int n = nc / Ca, c = nc % Ca;
    const size_t plane_off = ((size_t)n * C + c) * (size_t)H * (size_t)W;
    const T *xp = x + plane_off;
    T *op = out + plane_off;
    const int x0 = txi * kTileW, y0 = tyi * TH;

    // halo tile -> LDS, zero outside the image
    for (int idx = threadIdx.x; idx < HR * HC; idx += kThreads) {
        const int r = idx / HC, cc = idx - r * HC;
        const int gy = y0 - PH + r, gx = x0 - PH + cc;
        float v = 0.f;
        if (gy >= 0 && gy < H && gx >= 0 && gx < W) v = to_f32(xp[(size_t)gy * W + gx]);
        tile[r * PITCH + cc] = v;
    }
    __syncthreads();

    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const float *lkc = lk + (size_t)c * lk_cstride;

    float acc[RY][4];
#pragma unroll
    for (int oy = 0; oy < RY; ++oy)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[oy][q] = 0.f;

    const float *trow = tile + (ty * RY) * PITCH + 4 * tx;

    auto row_step = [&](int r) {
        float v[NV];
        if (OFF == 0) {
            const float4 *src = reinterpret_cast<const float4 *>(trow + r * PITCH);
#pragma unroll
            for (int k = 0; k < NV / 4; ++k) {
                float4 f = src[k];
                v[4 * k + 0] = f.x;
                v[4 * k + 1] = f.y;
                v[4 * k + 2] = f.z;
                v[4 * k + 3] = f.w;
            }
        } else {
            const float *src = trow + (r + OFF) * PITCH + OFF;
#pragma unroll
            for (int k = 0; k < NV; ++k) v[k] = k < KS + 3 ? src[k] : 0.f;
        }
#pragma unroll
        for (int oy = 0; oy < RY; ++oy) {
            const int i = r - oy;  // kernel row that maps tile row r to output row oy
            if (i >= 0 && i < KS) {
                const float *wrow = lkc + i * KS;
#pragma unroll
                for (int j = 0; j < KS; ++j) {
                    const float w = wrow[j];
#pragma unroll
                    for (int q = 0; q < 4; ++q) acc[oy][q] = fmaf(w, v[j + q], acc[oy][q]);
                }
            }
        }
    };

    if (kUnrollRows) {
#pragma unroll
        for (int r = 0; r < RY + KS - 1; ++r) row_step(r);
    } else {
#pragma unroll 1
        for (int r = 0; r < RY + KS - 1; ++r) row_step(r);
    }

    if (dk != nullptr) {
        const float *dkc = dk + ((size_t)n * Ca + c) * 9;
        float d[9];
#pragma unroll
        for (int k = 0; k < 9; ++k) d[k] = dkc[k];
#pragma unroll
        for (int r = 0; r < RY + 2; ++r) {
            float v[6];
            const float *src = trow + (r + PH - 1) * PITCH + (PH - 1);
#pragma unroll
            for (int k = 0; k < 6; ++k) v[k] = src[k];
#pragma unroll
            for (int oy = 0; oy < RY; ++oy) {
                const int i = r - oy;
                if (i >= 0 && i < 3) {
#pragma unroll
                    for (int j = 0; j < 3; ++j)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            acc[oy][q] = fmaf(d[i * 3 + j], v[j + q], acc[oy][q]);
                }
            }
        }
    }

    const int gx = x0 + 4 * tx;
#pragma unroll
    for (int oy = 0; oy < RY; ++oy) {
        const int gy = y0 + ty * RY + oy;
        if (gy >= H) continue;
        T *dst = op + (size_t)gy * W + gx;
        if (vec_ok && gx + 3 < W) {
            store4(dst, acc[oy]);
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (gx + q < W) store1(dst + q, acc[oy][q]);
        }
    }
}

// ---------------------------------------------------------------------------
// Pass-through of the identity channels (Eq. 4 lines 1 and 4): per image one
// contiguous byte range.  16-byte accesses when both sides allow it.
// ---------------------------------------------------------------------------
constexpr int kCopyVecPerThread = 4;
constexpr size_t kCopyChunk = (size_t)kThreads * 16 * kCopyVecPerThread;  // bytes per block

__global__ __launch_bounds__(kThreads) void copy_kernel(const char *__restrict__ x,
                                                        char *__restrict__ out, size_t img_bytes,
                                                        size_t off_bytes, size_t len_bytes,
                                                        int chunks_per_img, int vec_ok, int elem_bytes)
{
    const int n = blockIdx.x / chunks_per_img;
    const size_t chunk = (size_t)(blockIdx.x % chunks_per_img);
    const char *src = x + (size_t)n * img_bytes + off_bytes;
    char *dst = out + (size_t)n * img_bytes + off_bytes;
    const size_t begin = chunk * kCopyChunk;
    const size_t end = begin + kCopyChunk < len_bytes ? begin + kCopyChunk : len_bytes;
    if (vec_ok) {
        u32x4 v[kCopyVecPerThread];
#pragma unroll
        for (int k = 0; k < kCopyVecPerThread; ++k) {
            size_t o = begin + ((size_t)k * kThreads + threadIdx.x) * 16;
            if (o + 16 <= end) v[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + o));
        }
#pragma unroll
        for (int k = 0; k < kCopyVecPerThread; ++k) {
            size_t o = begin + ((size_t)k * kThreads + threadIdx.x) * 16;
            if (o + 16 <= end) __builtin_nontemporal_store(v[k], reinterpret_cast<u32x4 *>(dst + o));
        }
        // a range that is not a multiple of 16 bytes ends with whole elements
        const size_t tail = len_bytes & ~(size_t)15;
        if (end == len_bytes && tail < len_bytes) {
            size_t o = tail + (size_t)threadIdx.x * elem_bytes;
            if (o < len_bytes) {
                if (elem_bytes == 4)
                    *reinterpret_cast<uint32_t *>(dst + o) = *reinterpret_cast<const uint32_t *>(src + o);
                else
                    *reinterpret_cast<uint16_t *>(dst + o) = *reinterpret_cast<const uint16_t *>(src + o);
            }
        }
    } else {
        for (size_t o = begin + (size_t)threadIdx.x * elem_bytes; o < end; o += (size_t)kThreads * elem_bytes) {
            if (elem_bytes == 4)
                *reinterpret_cast<uint32_t *>(dst + o) = *reinterpret_cast<const uint32_t *>(src + o);
            else
                *reinterpret_cast<uint16_t *>(dst + o) = *reinterpret_cast<const uint16_t *>(src + o);
        }
    }
}

__global__ void fill_zero_kernel(uint32_t *p, size_t words)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < words) p[i] = 0u;
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
struct WsLayout {
    int nslab;
    size_t partials_off, dk_off, total;
};

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

bool ws_layout(int N, int Ca, int H, int W, WsLayout *l)
{
    if (N < 1 || Ca < 0 || H < 1 || W < 1) return false;
    const size_t hw = (size_t)H * (size_t)W;
    if (hw >= ((size_t)1 << 31)) return false;
    l->nslab = (int)((hw + kPoolSlab - 1) / kPoolSlab);
    size_t off = 0;
    l->partials_off = off;
    off = round_up(off + (size_t)N * Ca * l->nslab * sizeof(float), kWsAlign);
    l->dk_off = off;
    off = round_up(off + (size_t)N * Ca * 9 * sizeof(float), kWsAlign);
    l->total = off < kWsAlign ? kWsAlign : off;
    return true;
}

esc_status check_common(const void *x, esc_dtype dt, int N, int C, int H, int W, int Ca)
{
    if (dt != ESC_F32 && dt != ESC_BF16) return ESC_ERR_DTYPE;
    if (N < 1 || C < 1 || H < 1 || W < 1 || Ca < 0 || Ca > C) return ESC_ERR_SHAPE;
    if (x == nullptr) return ESC_ERR_NULL;
    if ((size_t)H * (size_t)W >= ((size_t)1 << 31)) return ESC_ERR_UNSUPPORTED;
    if (Ca > kMaxCa) return ESC_ERR_UNSUPPORTED;
    const size_t es = dt == ESC_F32 ? 4 : 2;
    if (((uintptr_t)x % es) != 0) return ESC_ERR_SHAPE;
    return ESC_OK;
}

esc_status check_gen(const esc_gen_params *gen, int Ca)
{
    if (gen->hidden < 0) return ESC_ERR_SHAPE;
    if (gen->hidden > kMaxHidden) return ESC_ERR_UNSUPPORTED;
    if (Ca > 0 && gen->w_up == nullptr) return ESC_ERR_NULL;
    if (Ca > 0 && gen->hidden > 0 && gen->w_down == nullptr) return ESC_ERR_NULL;
    return ESC_OK;
}

esc_status check_ws(void *ws, size_t ws_bytes, const WsLayout &l)
{
    if (ws == nullptr || ((uintptr_t)ws % kWsAlign) != 0 || ws_bytes < l.total) return ESC_ERR_WORKSPACE;
    return ESC_OK;
}

// blocks in a 1-D grid must stay below 2^31
bool grid_ok(size_t blocks) { return blocks > 0 && blocks < ((size_t)1 << 31); }

template <typename T>
esc_status launch_pool_gen(const T *x, int N, int C, int H, int W, int Ca, const esc_gen_params *gen,
                           float *partials, int nslab, float *dk, hipStream_t s)
{
    const size_t pool_blocks = (size_t)N * Ca * nslab;
    if (!grid_ok(pool_blocks)) return ESC_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(pool_kernel<T>, dim3((unsigned)pool_blocks), dim3(kThreads), 0, s, x, partials, C, Ca,
                       H * W, nslab);
    hipLaunchKernelGGL(gen_kernel, dim3((unsigned)N), dim3(kThreads), 0, s, partials, nslab,
                       (float)((double)H * (double)W), Ca, gen->hidden, gen->w_down, gen->b_down, gen->w_up,
                       gen->b_up, dk);
    return hipGetLastError() == hipSuccess ? ESC_OK : ESC_ERR_HIP;
}

int conv_ry_override()
{
    static int v = [] {
        const char *e = getenv("ESC_CONV_RY");
        return e ? atoi(e) : 0;
    }();
    return v;
}

template <int KS, int RY, typename T>
void launch_conv_one(const T *x, T *out, const float *lk, long lk_cstride, const float *dk, int N, int C,
                     int Ca, int H, int W, int vec_ok, hipStream_t s)
{
    const int tiles_x = (W + kTileW - 1) / kTileW;
    const int tiles_y = (H + 16 * RY - 1) / (16 * RY);
    const size_t blocks = (size_t)tiles_x * tiles_y * N * Ca;
    hipLaunchKernelGGL((conv_kernel<KS, RY, T>), dim3((unsigned)blocks), dim3(kThreads), 0, s, x, out, lk,
                       lk_cstride, dk, C, Ca, H, W, tiles_x, tiles_y, vec_ok);
}

template <int KS, typename T>
void launch_conv_ks(const T *x, T *out, const float *lk, long lk_cstride, const float *dk, int N, int C,
                    int Ca, int H, int W, int vec_ok, hipStream_t s)
{
    // taller register blocks once there is enough work to fill 256 CUs several times over
    const size_t tiles4 = (size_t)((W + kTileW - 1) / kTileW) * ((H + 63) / 64) * N * Ca;
    int ry = tiles4 >= 2048 ? 4 : 2;
    if (conv_ry_override() == 2 || conv_ry_override() == 4) ry = conv_ry_override();
    if (ry == 4)
        launch_conv_one<KS, 4, T>(x, out, lk, lk_cstride, dk, N, C, Ca, H, W, vec_ok, s);
    else
        launch_conv_one<KS, 2, T>(x, out, lk, lk_cstride, dk, N, C, Ca, H, W, vec_ok, s);
}

template <typename T>
esc_status launch_conv(const T *x, T *out, const float *lk, int Ks, long lk_cstride, const float *dk, int N,
                       int C, int Ca, int H, int W, int vec_ok, hipStream_t s)
{
    const size_t blocks2 = (size_t)((W + kTileW - 1) / kTileW) * ((H + 31) / 32) * N * Ca;
    if (!grid_ok(blocks2)) return ESC_ERR_UNSUPPORTED;
    switch (Ks) {
#define ESC_KS_CASE(K)                                                             \
    case K:                                                                        \
        launch_conv_ks<K, T>(x, out, lk, lk_cstride, dk, N, C, Ca, H, W, vec_ok, s); \
        break;
        ESC_KS_CASE(1)
        ESC_KS_CASE(3)
        ESC_KS_CASE(5)
        ESC_KS_CASE(7)
        ESC_KS_CASE(9)
        ESC_KS_CASE(11)
        ESC_KS_CASE(13)
        ESC_KS_CASE(15)
        ESC_KS_CASE(17)
        ESC_KS_CASE(19)
        ESC_KS_CASE(21)
        ESC_KS_CASE(23)
        ESC_KS_CASE(25)
        ESC_KS_CASE(27)
        ESC_KS_CASE(29)
        ESC_KS_CASE(31)
#undef ESC_KS_CASE
    default:
        return ESC_ERR_UNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? ESC_OK : ESC_ERR_HIP;
}

esc_status launch_copy(const void *x, void *out, esc_dtype dt, int N, int C, int H, int W, int Ca,
                       hipStream_t s)
{
    if (Ca >= C) return ESC_OK;
    const size_t es = dt == ESC_F32 ? 4 : 2;
    const size_t plane = (size_t)H * W * es;
    const size_t img_bytes = plane * C, off = plane * Ca, len = plane * (C - Ca);
    const size_t chunks = (len + kCopyChunk - 1) / kCopyChunk;
    if (!grid_ok(chunks * (size_t)N) || chunks >= ((size_t)1 << 31)) return ESC_ERR_UNSUPPORTED;
    const int vec_ok = ((uintptr_t)x % 16 == 0) && ((uintptr_t)out % 16 == 0) && (img_bytes % 16 == 0) &&
                       (off % 16 == 0);
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)(chunks * N)), dim3(kThreads), 0, s, (const char *)x,
                       (char *)out, img_bytes, off, len, (int)chunks, vec_ok, (int)es);
    return hipGetLastError() == hipSuccess ? ESC_OK : ESC_ERR_HIP;
}

}  // namespace

extern "C" {

size_t esc_workspace_bytes(int N, int C_a, int H, int W)
{
    WsLayout l;
    if (!ws_layout(N, C_a, H, W, &l)) return 0;
    return l.total;
}

esc_status esc_workspace_init(void *workspace, size_t workspace_bytes, void *stream)
{
    if (workspace == nullptr || ((uintptr_t)workspace % kWsAlign) != 0 || workspace_bytes < kWsAlign)
        return ESC_ERR_WORKSPACE;
    const size_t words = workspace_bytes / 4;
    const size_t blocks = (words + kThreads - 1) / kThreads;
    if (!grid_ok(blocks)) return ESC_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream,
                       (uint32_t *)workspace, words);
    return hipGetLastError() == hipSuccess ? ESC_OK : ESC_ERR_HIP;
}

esc_status esc_dynkernel_gen(const void *x, esc_dtype dt, int N, int C, int H, int W, int C_a,
                             const esc_gen_params *gen, float *dk_out, void *workspace,
                             size_t workspace_bytes, void *stream)
{
    esc_status st = check_common(x, dt, N, C, H, W, C_a);
    if (st != ESC_OK) return st;
    if (gen == nullptr) return ESC_ERR_NULL;
    if ((st = check_gen(gen, C_a)) != ESC_OK) return st;
    if (C_a > 0 && dk_out == nullptr) return ESC_ERR_NULL;
    WsLayout l;
    if (!ws_layout(N, C_a, H, W, &l)) return ESC_ERR_SHAPE;
    if ((st = check_ws(workspace, workspace_bytes, l)) != ESC_OK) return st;
    if (C_a == 0) return ESC_OK;
    float *partials = (float *)((char *)workspace + l.partials_off);
    if (dt == ESC_F32)
        return launch_pool_gen((const float *)x, N, C, H, W, C_a, gen, partials, l.nslab, dk_out,
                               (hipStream_t)stream);
    return launch_pool_gen((const bf16_t *)x, N, C, H, W, C_a, gen, partials, l.nslab, dk_out,
                           (hipStream_t)stream);
}

esc_status esc_convattn_forward(const void *x, esc_dtype dt, int N, int C, int H, int W, int C_a,
                                const float *lk, int Ks, long lk_channel_stride,
                                const esc_gen_params *gen, const float *dk_in, void *out,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    esc_status st = check_common(x, dt, N, C, H, W, C_a);
    if (st != ESC_OK) return st;
    if (out == nullptr) return ESC_ERR_NULL;
    if (Ks < 1 || (Ks % 2) == 0) return Ks < 1 ? ESC_ERR_SHAPE : ESC_ERR_UNSUPPORTED;
    if (Ks > kMaxKs) return ESC_ERR_UNSUPPORTED;
    if (C_a > 0 && lk == nullptr) return ESC_ERR_NULL;
    if (lk_channel_stride != 0 && lk_channel_stride < (long)Ks * Ks) return ESC_ERR_SHAPE;
    if (gen != nullptr && (st = check_gen(gen, C_a)) != ESC_OK) return st;
    const size_t es = dt == ESC_F32 ? 4 : 2;
    if (((uintptr_t)out % es) != 0) return ESC_ERR_SHAPE;
    const size_t bytes = (size_t)N * C * H * W * es;
    const uintptr_t xa = (uintptr_t)x, oa = (uintptr_t)out;
    if (xa < oa + bytes && oa < xa + bytes) return ESC_ERR_ALIAS;
    WsLayout l;
    if (!ws_layout(N, C_a, H, W, &l)) return ESC_ERR_SHAPE;
    if (gen != nullptr && (st = check_ws(workspace, workspace_bytes, l)) != ESC_OK) return st;

    hipStream_t s = (hipStream_t)stream;
    if (C_a > 0) {
        const float *dk = dk_in;
        float *partials = (float *)((char *)workspace + l.partials_off);
        float *dk_ws = (float *)((char *)workspace + l.dk_off);
        if (gen != nullptr) {
            st = dt == ESC_F32 ? launch_pool_gen((const float *)x, N, C, H, W, C_a, gen, partials, l.nslab,
                                                 dk_ws, s)
                               : launch_pool_gen((const bf16_t *)x, N, C, H, W, C_a, gen, partials, l.nslab,
                                                 dk_ws, s);
            if (st != ESC_OK) return st;
            dk = dk_ws;
        }
        // 16-byte (fp32) / 8-byte (bf16) row stores need W % 4 == 0 and an aligned base
        const int vec_ok = (W % 4 == 0) && ((uintptr_t)out % (4 * es) == 0);
        st = dt == ESC_F32 ? launch_conv((const float *)x, (float *)out, lk, Ks, lk_channel_stride, dk, N, C,
                                         C_a, H, W, vec_ok, s)
                           : launch_conv((const bf16_t *)x, (bf16_t *)out, lk, Ks, lk_channel_stride, dk, N,
                                         C, C_a, H, W, vec_ok, s);
        if (st != ESC_OK) return st;
    }
    return launch_copy(x, out, dt, N, C, H, W, C_a, s);
}

const char *esc_status_string(esc_status s)
{
    switch (s) {
    case ESC_OK: return "ok";
    case ESC_ERR_NULL: return "a required pointer is NULL";
    case ESC_ERR_SHAPE: return "a size or stride is out of its domain";
    case ESC_ERR_DTYPE: return "unknown storage type";
    case ESC_ERR_UNSUPPORTED: return "outside the library's limits (Ks odd <= 31, C_a <= 256, hidden <= 256)";
    case ESC_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case ESC_ERR_ALIAS: return "out overlaps x";
    case ESC_ERR_HIP: return "the HIP runtime refused a launch";
    }
    return "unknown status";
}

}  // extern "C"

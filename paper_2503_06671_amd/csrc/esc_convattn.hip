// ConvAttn forward for gfx950 (MI355X): hand-written HIP kernels and the C ABI
// declared in include/esc_convattn.h.
//
// The operation is Eq. 4 of the ESC paper with the depth-wise large kernel of
// the paragraph around Eq. 5.  Everything is plain fp32 vector arithmetic (a
// depth-wise convolution has no reduction shared between outputs, so there is
// nothing to feed a matrix core with).
//
// One launch does the whole forward.  The work is cut into items that blocks take
// from a queue in this order:
//
//   pool items   GAP partial sums of the attention slice, one 4096-element slab each
//   gen items    one per image: finish the GAP, run the kernel estimator, publish DK
//   conv items   one 64 x (16*RY) output tile of one (image, channel) plane: LK taps
//                from an LDS halo tile, then DK's nine taps once DK is published
//   copy items   16 KiB of the identity channels (interleaved with the conv items so
//                streaming and arithmetic overlap on every compute unit)
//
// A block's first item is its block index; further items come from an atomic
// counter.  An item only ever waits for items with smaller indices (conv -> gen ->
// pool), and pool items wait for nothing, so every wait ends as long as the blocks
// of the grid are co-resident (the host sizes the grid to the occupancy limit) -
// and each wait is bounded anyway: on expiry the block raises the error word of the
// workspace and goes on.
//
// Blocks talk through 64-bit mailboxes {fp32 value, 32-bit call tag} written and
// read with relaxed device-scope atomics.  A mailbox is valid when its tag equals
// the tag of this call, so nothing has to be cleared between calls and no fence
// (and no cache write-back) is needed: each datum validates itself.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include <atomic>

#include "esc_convattn.h"

namespace {

constexpr int kThreads = 256;      // 4 wavefronts per block
constexpr int kTileW = 64;         // conv tile width: 16 lanes x 4 outputs
constexpr int kPoolSlab = 4096;    // elements per GAP partial sum
constexpr int kMaxCa = 256;
constexpr int kMaxHidden = 256;
constexpr int kMaxKs = 31;
constexpr size_t kWsAlign = 256;
constexpr unsigned kSpinLimit = 1u << 20;  // bounded wait: seconds, far beyond any real wait
constexpr int kCopyVecPerThread = 4;
constexpr size_t kCopyChunk = (size_t)kThreads * 16 * kCopyVecPerThread;  // bytes per copy item

struct bf16_t {
    uint16_t bits;
};
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned long long u64;

// ---------------------------------------------------------------------------
// storage helpers
// ---------------------------------------------------------------------------
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
// mailboxes
// ---------------------------------------------------------------------------
__device__ __forceinline__ void box_put(u64 *box, float v, uint32_t tag)
{
    __hip_atomic_store(box, ((u64)tag << 32) | (u64)__float_as_uint(v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}

// Waits (bounded) until the mailbox carries this call's tag.  On expiry raises *err.
__device__ __forceinline__ float box_get(const u64 *box, uint32_t tag, unsigned *err)
{
    for (unsigned spin = 0; spin < kSpinLimit; ++spin) {
        const u64 v = __hip_atomic_load(box, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((uint32_t)(v >> 32) == tag) return __uint_as_float((uint32_t)v);
        __builtin_amdgcn_s_sleep(4);
    }
    __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return 0.f;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

// ---------------------------------------------------------------------------
// kernel arguments
// ---------------------------------------------------------------------------
struct FwdParams {
    const void *x;
    void *out;
    const float *lk;
    long lk_cstride;
    const float *dk_in;  // DK given by the caller (no estimator), or NULL
    float *dk_out;       // esc_dynkernel_gen: where the estimator's DK goes, else NULL
    const float *w_down, *b_down, *w_up, *b_up;
    int hidden;
    int has_gen;         // pool + gen items exist; conv items wait for the DK mailboxes
    int N, C, Ca, H, W;
    int nslab;           // pool slabs per (image, channel) plane
    float hw;            // H*W as a float, the GAP divisor
    int tiles_x, tiles_y;
    unsigned n_pool, n_gen, n_conv, n_copy;  // item counts
    unsigned copy_chunks;                    // copy items per image
    size_t img_bytes, idt_off, idt_len;      // pass-through range of one image, in bytes
    int conv_vec_ok, copy_vec_ok, pool_vec_ok, elem_bytes;
    u64 *pool_box;       // [N*Ca*nslab] partial sums
    u64 *dk_box;         // [N*Ca*9]
    u64 *queue;          // work counter {tag, next item}
    unsigned *err;
    uint32_t tag;
};

// ---------------------------------------------------------------------------
// pool item (Eq. 4 line 2, first half).  Thread t adds elements
// base + (k*256 + t)*V + q for k, then q, ascending - the same order whether the
// 16-byte loads are usable or not - then a fixed tree over the block.  The
// decomposition depends on H*W only, so a batch reproduces its images run alone.
// ---------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void pool_item(const FwdParams &p, unsigned item, float *s_red)
{
    constexpr int V = 16 / (int)sizeof(T);  // elements per 16-byte load
    constexpr int K = kPoolSlab / (kThreads * V);
    const int HW = p.H * p.W;
    const unsigned nc = item / (unsigned)p.nslab;
    const int slab = (int)(item - nc * (unsigned)p.nslab);
    const int n = (int)(nc / (unsigned)p.Ca), c = (int)(nc % (unsigned)p.Ca);
    const T *plane = (const T *)p.x + ((size_t)n * p.C + c) * (size_t)HW;
    const int base = slab * kPoolSlab;
    float s = 0.f;
    if (p.pool_vec_ok && base + kPoolSlab <= HW) {
        u32x4 raw[K];
#pragma unroll
        for (int k = 0; k < K; ++k)
            raw[k] = *reinterpret_cast<const u32x4 *>(plane + base + (k * kThreads + (int)threadIdx.x) * V);
#pragma unroll
        for (int k = 0; k < K; ++k) {
            if (sizeof(T) == 4) {
#pragma unroll
                for (int q = 0; q < 4; ++q) s += __uint_as_float(raw[k][q]);
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    s += __uint_as_float(raw[k][q] << 16);
                    s += __uint_as_float(raw[k][q] & 0xffff0000u);
                }
            }
        }
    } else {
#pragma unroll
        for (int k = 0; k < K; ++k)
#pragma unroll
            for (int q = 0; q < V; ++q) {
                const int idx = base + (k * kThreads + (int)threadIdx.x) * V + q;
                if (idx < HW) s += to_f32(plane[idx]);
            }
    }
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = s_red[0];
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) t += s_red[w];
        box_put(p.pool_box + item, t, p.tag);
    }
}

// ---------------------------------------------------------------------------
// gen item (Eq. 4 line 2, second half): image n.  Wavefront w finishes the GAP
// of channels w, w+4, ...: lane l adds slabs l, l+64, ... in order, then the
// wavefront tree.  Then the estimator, one output per thread.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float gelu_erf(float v)
{
    return 0.5f * v * (1.f + erff(v * 0.70710678118654752440f));
}

__device__ __forceinline__ void gen_item(const FwdParams &p, unsigned n, float *s_g, float *s_t)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int c = wave; c < p.Ca; c += kThreads / 64) {
        const u64 *boxes = p.pool_box + ((size_t)n * p.Ca + c) * p.nslab;
        float s = 0.f;
        for (int k = lane; k < p.nslab; k += 64) s += box_get(boxes + k, p.tag, p.err);
        s = wave_sum(s);
        if (lane == 0) s_g[c] = s / p.hw;
    }
    __syncthreads();
    const float *in = s_g;
    int K = p.Ca;
    if (p.hidden > 0) {
        for (int m = threadIdx.x; m < p.hidden; m += kThreads) {
            float s = p.b_down ? p.b_down[m] : 0.f;
            for (int k = 0; k < p.Ca; ++k) s = fmaf(p.w_down[(size_t)m * p.Ca + k], s_g[k], s);
            s_t[m] = gelu_erf(s);
        }
        __syncthreads();
        in = s_t;
        K = p.hidden;
    }
    for (int o = threadIdx.x; o < 9 * p.Ca; o += kThreads) {
        float s = p.b_up ? p.b_up[o] : 0.f;
        for (int k = 0; k < K; ++k) s = fmaf(p.w_up[(size_t)o * K + k], in[k], s);
        const size_t idx = (size_t)n * 9 * p.Ca + o;
        box_put(p.dk_box + idx, s, p.tag);
        if (p.dk_out) p.dk_out[idx] = s;
    }
}

// ---------------------------------------------------------------------------
// conv item (Eq. 4 line 3).  The zero-extended halo tile sits in LDS as fp32;
// thread (tx, ty) produces outputs x = 4*tx..4*tx+3 of rows ty*RY..ty*RY+RY-1.
// Each LDS row segment it loads (KS+3 values, 16-byte reads) feeds up to RY kernel
// rows, and the kernel weights are wave-uniform, so the tap loop is FMA with a
// scalar-register multiplier.  DK's nine taps run afterwards from the same tile,
// which is the only part that has to wait for the estimator.
// ---------------------------------------------------------------------------
template <int KS, int RY>
struct ConvGeom {
    static constexpr int P = (KS - 1) / 2;
    static constexpr int PH = P > 1 ? P : 1;  // halo width: DK's 3x3 needs one pixel even when Ks == 1
    static constexpr int OFF = PH - P;        // where the LK window starts inside the halo
    static constexpr int TH = 16 * RY;
    static constexpr int HR = TH + 2 * PH;
    static constexpr int HC = kTileW + 2 * PH;
    static constexpr int PITCH = (HC + 3) & ~3;
    static constexpr int NV = (KS + 3 + 3) & ~3;  // values a thread reads per tile row
    static constexpr int LDS_FLOATS = HR * PITCH;
};

template <int KS, int RY, typename T>
__device__ __forceinline__ void conv_item(const FwdParams &p, unsigned item, float *tile, float *s_dk)
{
    using G = ConvGeom<KS, RY>;
    constexpr int PH = G::PH, OFF = G::OFF, TH = G::TH, HR = G::HR, HC = G::HC, PITCH = G::PITCH,
                  NV = G::NV;
    constexpr bool kUnrollRows = (KS <= 13);
    const int H = p.H, W = p.W;

    unsigned b = item;
    const int txi = (int)(b % (unsigned)p.tiles_x);
    b /= (unsigned)p.tiles_x;
    const int tyi = (int)(b % (unsigned)p.tiles_y);
    const unsigned nc = b / (unsigned)p.tiles_y;
    const int n = (int)(nc / (unsigned)p.Ca), c = (int)(nc % (unsigned)p.Ca);
    const size_t plane_off = ((size_t)n * p.C + c) * (size_t)H * (size_t)W;
    const T *xp = (const T *)p.x + plane_off;
    T *op = (T *)p.out + plane_off;
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
    const float *lkc = p.lk + (size_t)c * p.lk_cstride;

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

    if (p.has_gen || p.dk_in != nullptr) {
        const size_t dk_idx = ((size_t)n * p.Ca + c) * 9;
        if (threadIdx.x < 9)
            s_dk[threadIdx.x] = p.has_gen ? box_get(p.dk_box + dk_idx + threadIdx.x, p.tag, p.err)
                                          : p.dk_in[dk_idx + threadIdx.x];
        __syncthreads();
        float d[9];
#pragma unroll
        for (int k = 0; k < 9; ++k) d[k] = s_dk[k];
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
        if (p.conv_vec_ok && gx + 3 < W) {
            store4(dst, acc[oy]);
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (gx + q < W) store1(dst + q, acc[oy][q]);
        }
    }
}

// ---------------------------------------------------------------------------
// copy item (Eq. 4 lines 1 and 4): 16 KiB of one image's identity channels,
// streamed with 16-byte non-temporal accesses when both sides allow it.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void copy_item(const FwdParams &p, unsigned item)
{
    const unsigned n = item / p.copy_chunks;
    const size_t chunk = (size_t)(item - n * p.copy_chunks);
    const char *src = (const char *)p.x + (size_t)n * p.img_bytes + p.idt_off;
    char *dst = (char *)p.out + (size_t)n * p.img_bytes + p.idt_off;
    const size_t len = p.idt_len;
    const size_t begin = chunk * kCopyChunk;
    const size_t end = begin + kCopyChunk < len ? begin + kCopyChunk : len;
    const int eb = p.elem_bytes;
    if (p.copy_vec_ok) {
        u32x4 v[kCopyVecPerThread];
#pragma unroll
        for (int k = 0; k < kCopyVecPerThread; ++k) {
            const size_t o = begin + ((size_t)k * kThreads + threadIdx.x) * 16;
            if (o + 16 <= end) v[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + o));
        }
#pragma unroll
        for (int k = 0; k < kCopyVecPerThread; ++k) {
            const size_t o = begin + ((size_t)k * kThreads + threadIdx.x) * 16;
            if (o + 16 <= end) __builtin_nontemporal_store(v[k], reinterpret_cast<u32x4 *>(dst + o));
        }
        // a range that is not a multiple of 16 bytes ends with whole elements
        const size_t tail = len & ~(size_t)15;
        if (end == len && tail < len) {
            const size_t o = tail + (size_t)threadIdx.x * eb;
            if (o < len) {
                if (eb == 4)
                    *reinterpret_cast<uint32_t *>(dst + o) = *reinterpret_cast<const uint32_t *>(src + o);
                else
                    *reinterpret_cast<uint16_t *>(dst + o) = *reinterpret_cast<const uint16_t *>(src + o);
            }
        }
    } else {
        for (size_t o = begin + (size_t)threadIdx.x * eb; o < end; o += (size_t)kThreads * eb) {
            if (eb == 4)
                *reinterpret_cast<uint32_t *>(dst + o) = *reinterpret_cast<const uint32_t *>(src + o);
            else
                *reinterpret_cast<uint16_t *>(dst + o) = *reinterpret_cast<const uint16_t *>(src + o);
        }
    }
}

// ---------------------------------------------------------------------------
// the one kernel.  KS == 0 builds the variant without conv items (used by
// esc_dynkernel_gen and for C_a == 0).
// ---------------------------------------------------------------------------
template <int KS, int RY, typename T>
__global__ __launch_bounds__(kThreads) void forward_kernel(const FwdParams p)
{
    constexpr int kTileFloats = ConvGeom<(KS > 0 ? KS : 1), RY>::LDS_FLOATS;
    __shared__ __align__(16) float tile[KS > 0 ? kTileFloats : 4];
    __shared__ float s_g[kMaxCa];
    __shared__ float s_t[kMaxHidden];
    __shared__ float s_small[16];
    __shared__ unsigned s_next;

    const unsigned first_mixed = p.n_pool + p.n_gen;
    const unsigned n_mixed = p.n_conv + p.n_copy;
    const unsigned total = first_mixed + n_mixed;
    unsigned item = blockIdx.x;
    while (item < total) {
        // take the next item now so the atomic's round trip hides behind this item's work
        unsigned next = 0;
        if (threadIdx.x == 0) {
            const u64 base = ((u64)p.tag << 32) | (u64)gridDim.x;
            __hip_atomic_fetch_max(p.queue, base, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            next = (unsigned)__hip_atomic_fetch_add(p.queue, (u64)1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (item < p.n_pool) {
            pool_item<T>(p, item, s_small);
        } else if (item < first_mixed) {
            gen_item(p, item - p.n_pool, s_g, s_t);
        } else {
            // conv and copy items alternate in proportion: mixed item j is a conv item
            // when floor((j+1)*n_conv/n_mixed) steps past floor(j*n_conv/n_mixed)
            const u64 j = item - first_mixed;
            const unsigned cb = (unsigned)(j * p.n_conv / n_mixed);
            const unsigned ca = (unsigned)((j + 1) * p.n_conv / n_mixed);
            if (ca > cb) {
                if constexpr (KS > 0) conv_item<KS, RY, T>(p, cb, tile, s_small);
            } else {
                copy_item(p, (unsigned)j - cb);
            }
        }
        if (threadIdx.x == 0) s_next = next;
        __syncthreads();
        item = s_next;
        __syncthreads();
    }
}

__global__ void fill_zero_kernel(uint32_t *ptr, size_t words)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < words) ptr[i] = 0u;
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
struct WsLayout {
    int nslab;
    size_t ctl_off, pool_off, dk_off, total;
};

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

bool ws_layout(int N, int Ca, int H, int W, WsLayout *l)
{
    if (N < 1 || Ca < 0 || H < 1 || W < 1) return false;
    const size_t hw = (size_t)H * (size_t)W;
    if (hw >= ((size_t)1 << 31)) return false;
    l->nslab = (int)((hw + kPoolSlab - 1) / kPoolSlab);
    size_t off = 0;
    l->ctl_off = off;  // [0] work counter, [1] error word
    off = round_up(off + 2 * sizeof(u64), kWsAlign);
    l->pool_off = off;
    off = round_up(off + (size_t)N * Ca * l->nslab * sizeof(u64), kWsAlign);
    l->dk_off = off;
    off = round_up(off + (size_t)N * Ca * 9 * sizeof(u64), kWsAlign);
    l->total = off;
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

esc_status check_ws(const void *ws, size_t ws_bytes, size_t need)
{
    if (ws == nullptr || ((uintptr_t)ws % kWsAlign) != 0 || ws_bytes < need) return ESC_ERR_WORKSPACE;
    return ESC_OK;
}

// every call gets its own non-zero tag; a zeroed workspace never matches one
uint32_t next_tag()
{
    static std::atomic<uint32_t> counter{0};
    uint32_t t;
    do {
        t = counter.fetch_add(1, std::memory_order_relaxed) + 1;
    } while (t == 0);
    return t;
}

int conv_ry_override()
{
    static int v = [] {
        const char *e = getenv("ESC_CONV_RY");
        return e ? atoi(e) : 0;
    }();
    return v;
}

int device_cus()
{
    static int cus = [] {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            return prop.multiProcessorCount;
        return 0;
    }();
    return cus;
}

template <int KS, int RY, typename T>
esc_status launch_variant(FwdParams &p, hipStream_t s)
{
    // blocks that can be resident at once: occupancy of this instantiation x compute units
    static int per_cu = 0;
    if (per_cu == 0) {
        int v = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&v, forward_kernel<KS, RY, T>, kThreads, 0) !=
                hipSuccess ||
            v < 1)
            return ESC_ERR_HIP;
        per_cu = v;
    }
    const int cus = device_cus();
    if (cus < 1) return ESC_ERR_HIP;
    const u64 total = (u64)p.n_pool + p.n_gen + p.n_conv + p.n_copy;
    if (total == 0) return ESC_OK;
    const u64 cap = (u64)per_cu * (u64)cus;
    const unsigned grid = (unsigned)(total < cap ? total : cap);
    hipLaunchKernelGGL((forward_kernel<KS, RY, T>), dim3(grid), dim3(kThreads), 0, s, p);
    return hipGetLastError() == hipSuccess ? ESC_OK : ESC_ERR_HIP;
}

template <int KS, typename T>
esc_status launch_ks(FwdParams &p, hipStream_t s)
{
    if constexpr (KS == 0) {
        return launch_variant<0, 2, T>(p, s);
    } else {
        // taller register blocks once there is enough work to fill the chip several times over
        const size_t tiles4 = (size_t)((p.W + kTileW - 1) / kTileW) * ((p.H + 63) / 64) * p.N * p.Ca;
        int ry = (tiles4 >= 2048 && KS <= 17) ? 4 : 2;
        if (conv_ry_override() == 2 || (conv_ry_override() == 4 && KS <= 17)) ry = conv_ry_override();
        const int th = 16 * ry;
        p.tiles_x = (p.W + kTileW - 1) / kTileW;
        p.tiles_y = (p.H + th - 1) / th;
        const size_t n_conv = (size_t)p.tiles_x * p.tiles_y * p.N * p.Ca;
        if (n_conv >= ((size_t)1 << 30)) return ESC_ERR_UNSUPPORTED;
        p.n_conv = (unsigned)n_conv;
        if constexpr (KS <= 17) {
            if (ry == 4) return launch_variant<KS, 4, T>(p, s);
        }
        return launch_variant<KS, 2, T>(p, s);
    }
}

template <typename T>
esc_status launch_typed(FwdParams &p, int Ks, hipStream_t s)
{
    switch (Ks) {
#define ESC_KS_CASE(K) \
    case K: return launch_ks<K, T>(p, s);
        ESC_KS_CASE(0)
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
    default: return ESC_ERR_UNSUPPORTED;
    }
}

// fills the parts of FwdParams every entry point shares
esc_status setup_common(FwdParams &p, const void *x, esc_dtype dt, int N, int C, int H, int W, int Ca,
                        const esc_gen_params *gen, void *workspace, const WsLayout &l)
{
    p = FwdParams{};
    p.x = x;
    p.N = N;
    p.C = C;
    p.Ca = Ca;
    p.H = H;
    p.W = W;
    p.nslab = l.nslab;
    p.hw = (float)((double)H * (double)W);
    p.elem_bytes = dt == ESC_F32 ? 4 : 2;
    p.tag = next_tag();
    if (gen != nullptr && Ca > 0) {
        p.has_gen = 1;
        p.hidden = gen->hidden;
        p.w_down = gen->w_down;
        p.b_down = gen->b_down;
        p.w_up = gen->w_up;
        p.b_up = gen->b_up;
        const size_t n_pool = (size_t)N * Ca * l.nslab;
        if (n_pool >= ((size_t)1 << 30)) return ESC_ERR_UNSUPPORTED;
        p.n_pool = (unsigned)n_pool;
        p.n_gen = (unsigned)N;
        const size_t plane_bytes = (size_t)H * W * p.elem_bytes;
        p.pool_vec_ok = ((uintptr_t)x % 16 == 0) && (plane_bytes % 16 == 0);
    }
    char *w = (char *)workspace;
    p.queue = (u64 *)(w + l.ctl_off);
    p.err = (unsigned *)(w + l.ctl_off + sizeof(u64));
    p.pool_box = (u64 *)(w + l.pool_off);
    p.dk_box = (u64 *)(w + l.dk_off);
    return ESC_OK;
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
    esc_status st = check_ws(workspace, workspace_bytes, kWsAlign);
    if (st != ESC_OK) return st;
    const size_t words = workspace_bytes / 4;
    const size_t blocks = (words + kThreads - 1) / kThreads;
    if (blocks >= ((size_t)1 << 31)) return ESC_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream,
                       (uint32_t *)workspace, words);
    return hipGetLastError() == hipSuccess ? ESC_OK : ESC_ERR_HIP;
}

esc_status esc_workspace_errors(const void *workspace, size_t workspace_bytes, void *stream,
                                unsigned *errors_out)
{
    if (errors_out == nullptr) return ESC_ERR_NULL;
    esc_status st = check_ws(workspace, workspace_bytes, kWsAlign);
    if (st != ESC_OK) return st;
    unsigned v = 0;
    if (hipMemcpyAsync(&v, (const char *)workspace + sizeof(u64), sizeof v, hipMemcpyDeviceToHost,
                       (hipStream_t)stream) != hipSuccess)
        return ESC_ERR_HIP;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return ESC_ERR_HIP;
    *errors_out = v;
    return ESC_OK;
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
    if ((st = check_ws(workspace, workspace_bytes, l.total)) != ESC_OK) return st;
    if (C_a == 0) return ESC_OK;
    FwdParams p;
    if ((st = setup_common(p, x, dt, N, C, H, W, C_a, gen, workspace, l)) != ESC_OK) return st;
    p.dk_out = dk_out;
    return dt == ESC_F32 ? launch_typed<float>(p, 0, (hipStream_t)stream)
                         : launch_typed<bf16_t>(p, 0, (hipStream_t)stream);
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
    if ((st = check_ws(workspace, workspace_bytes, l.total)) != ESC_OK) return st;

    FwdParams p;
    if ((st = setup_common(p, x, dt, N, C, H, W, C_a, gen, workspace, l)) != ESC_OK) return st;
    p.out = out;
    p.lk = lk;
    p.lk_cstride = lk_channel_stride;
    p.dk_in = (gen == nullptr && C_a > 0) ? dk_in : nullptr;
    // 16-byte (fp32) / 8-byte (bf16) row stores need W % 4 == 0 and an aligned base
    p.conv_vec_ok = (W % 4 == 0) && ((uintptr_t)out % (4 * es) == 0);
    if (C_a < C) {
        const size_t plane = (size_t)H * W * es;
        p.img_bytes = plane * C;
        p.idt_off = plane * C_a;
        p.idt_len = plane * (C - C_a);
        const size_t chunks = (p.idt_len + kCopyChunk - 1) / kCopyChunk;
        if (chunks * (size_t)N >= ((size_t)1 << 30)) return ESC_ERR_UNSUPPORTED;
        p.copy_chunks = (unsigned)chunks;
        p.n_copy = (unsigned)(chunks * N);
        p.copy_vec_ok = (xa % 16 == 0) && (oa % 16 == 0) && (p.img_bytes % 16 == 0) && (p.idt_off % 16 == 0);
    }
    const int ks_variant = C_a > 0 ? Ks : 0;
    return dt == ESC_F32 ? launch_typed<float>(p, ks_variant, (hipStream_t)stream)
                         : launch_typed<bf16_t>(p, ks_variant, (hipStream_t)stream);
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

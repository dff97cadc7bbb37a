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
//   gen items    one per image, only when an image has many slabs: finish the GAP,
//                run the kernel estimator, publish DK
//   conv items   one 64 x (16*RY) output tile of one (image, channel) plane: LK taps
//                from an LDS halo tile with the channel's weights staged in LDS, then
//                DK's nine taps once DK is known
//   copy items   16 KiB of the identity channels, interleaved with the conv items so
//                streaming and arithmetic overlap on every compute unit
//
// Block b takes items b, b + grid, b + 2*grid, ...  An item only ever waits for
// items with smaller indices (conv -> gen -> pool), pool items wait for nothing and
// come first in every block's list, so every wait ends as long as the blocks of the
// grid are co-resident (the host sizes the grid to what the kernel is compiled to
// fit) - and each wait is bounded anyway: on expiry the block raises the error word
// of the workspace and goes on.  The grid size is kept coprime with the length of
// the conv/copy pattern so that every block meets both kinds of item.
//
// Blocks talk through 64-bit mailboxes {fp32 value, 32-bit call tag} written and
// read with relaxed device-scope atomics.  A mailbox is valid when its tag equals
// the tag of this call, so nothing has to be cleared between calls and no fence
// (and no cache write-back) is needed: each datum validates itself.  The tag is a
// call counter kept in the workspace, one copy per group of blocks (block index
// modulo 64): a block reads its group's copy, and the last block of a group to
// announce that it is leaving advances that copy.  Every copy advances exactly once
// per call, so all agree at every launch, no address is hot, and a captured launch
// can be replayed any number of times.
//
// Three facts about the machine shape the code (measured, not assumed):
//   - an FMA whose multiplier sits in a scalar register issues at half the rate of
//     one with both operands in vector registers, so the tap weights are read from
//     LDS (a broadcast read) into vector registers;
//   - vector-memory results return in order, so an atomic with a slow answer delays
//     every later load of its wavefront: the leave announcement is issued after an
//     item's loads, by a wavefront that polls no mailbox afterwards;
//   - a thousand atomics on one address take tens of microseconds: nothing here
//     has more than a handful of blocks on the same word.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "esc_convattn.h"

namespace {

constexpr int kThreads = 256;      // 4 wavefronts per block
constexpr int kTileW = 64;         // conv tile width: 16 lanes x 4 outputs
constexpr int kPoolSlab = 4096;    // elements per GAP partial sum
constexpr int kMaxCa = 256;
constexpr int kMaxHidden = 256;
constexpr int kMaxKs = 31;
constexpr size_t kWsAlign = 256;
constexpr unsigned kSpinLimit = 1u << 20;  // bounded wait: about a second, far beyond any real wait
constexpr int kBlocksPerCu = 4;    // resident blocks per compute unit the kernel is compiled for (<= 128 VGPRs)
constexpr int kCopyVecPerThread = 4;
constexpr size_t kCopyChunk = (size_t)kThreads * 16 * kCopyVecPerThread;  // bytes per copy item
constexpr int kStage = 1024;       // pool mailboxes staged in LDS per round (multiple of 64)
constexpr int kPollThreads = 192;  // wavefronts 0-2 poll mailboxes; wavefront 3 carries the leave atomic
constexpr int kStagePerThread = (kStage + kPollThreads - 1) / kPollThreads;
constexpr int kGroups = 64;        // block groups with their own call counter and leave counter
constexpr int kCtlStride = 16;     // 32-bit words between two groups' counters (one 64-byte line each)

struct bf16_t {
    uint16_t bits;
};
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned long long u64;

// Optional per-item timeline (development builds only, -DESC_TRACE): 16 words per item.
#ifdef ESC_TRACE
#define ESC_STAMP(rec, k)                                                    \
    do {                                                                     \
        if ((rec) != nullptr && threadIdx.x == 0) (rec)[k] = wall_clock64(); \
    } while (0)
#else
#define ESC_STAMP(rec, k) \
    do {                  \
    } while (0)
#endif

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

// four consecutive elements from an address aligned to all four
__device__ __forceinline__ void load4(const float *p, float *v)
{
    const float4 f = *reinterpret_cast<const float4 *>(p);
    v[0] = f.x;
    v[1] = f.y;
    v[2] = f.z;
    v[3] = f.w;
}
__device__ __forceinline__ void load4(const bf16_t *p, float *v)
{
    const uint2 w = *reinterpret_cast<const uint2 *>(p);
    v[0] = __uint_as_float(w.x << 16);
    v[1] = __uint_as_float(w.x & 0xffff0000u);
    v[2] = __uint_as_float(w.y << 16);
    v[3] = __uint_as_float(w.y & 0xffff0000u);
}

// x / d for x < 2^31 by multiply-high and shift (host fills mul and shift)
struct FastDiv {
    uint32_t d, mul, shift;
};
__device__ __forceinline__ uint32_t fdiv(uint32_t x, const FastDiv &f)
{
    return (__umulhi(x, f.mul) + x) >> f.shift;
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
        __builtin_amdgcn_s_sleep(2);
    }
    __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return 0.f;
}

// Whole block: waits for cnt (<= kStage) consecutive mailboxes and copies their values to
// dst[0..cnt).  A thread's polls are issued together so their round trips overlap.
__device__ __forceinline__ void boxes_to_lds(const u64 *boxes, int cnt, float *dst, uint32_t tag, unsigned *err)
{
    bool pend[kStagePerThread];
#pragma unroll
    for (int u = 0; u < kStagePerThread; ++u)
        pend[u] = threadIdx.x < kPollThreads && (int)threadIdx.x + u * kPollThreads < cnt;
    bool any = false;
    for (unsigned spin = 0; spin < kSpinLimit; ++spin) {
        u64 v[kStagePerThread];
#pragma unroll
        for (int u = 0; u < kStagePerThread; ++u)
            if (pend[u])
                v[u] = __hip_atomic_load(boxes + threadIdx.x + u * kPollThreads, __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
        any = false;
#pragma unroll
        for (int u = 0; u < kStagePerThread; ++u)
            if (pend[u]) {
                if ((uint32_t)(v[u] >> 32) == tag) {
                    dst[threadIdx.x + u * kPollThreads] = __uint_as_float((uint32_t)v[u]);
                    pend[u] = false;
                } else {
                    any = true;
                }
            }
        if (!any) break;
        __builtin_amdgcn_s_sleep(2);
    }
    if (any) __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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
enum : int {
    kDkNone = 0,    // DK = 0
    kDkGiven = 1,   // caller's dk_in
    kDkBoxes = 2,   // published by a gen item
    kDkDirect = 3   // each conv item finishes the GAP and runs its nine estimator outputs itself
};
constexpr int kDirectMaxBoxes = 512;  // direct mode while C_a * nslab mailboxes stay this few

struct FwdParams {
    const void *x;
    void *out;
    const float *lk;
    long lk_cstride;
    const float *dk_in;  // DK given by the caller (no estimator), or NULL
    float *dk_out;       // esc_dynkernel_gen: where the estimator's DK goes, else NULL
    const float *w_down, *b_down, *w_up, *b_up;
    int hidden;
    int dk_mode;         // where conv items take DK from (kDk*)
    int N, C, Ca, H, W;
    int nslab;           // pool slabs per (image, channel) plane
    float hw;            // H*W as a float, the GAP divisor
    unsigned n_pool, n_gen, n_conv, n_copy;  // item counts
    // conv and copy items alternate in groups of mix_a conv + mix_b copy items while both
    // last (mix_groups groups); the rest of the conv items follow, then the rest of the copy items
    unsigned mix_a, mix_b, mix_groups;
    FastDiv div_nslab, div_ca, div_tiles_x, div_tiles_y, div_chunks, div_mix;
    size_t img_bytes, idt_off, idt_len;      // pass-through range of one image, in bytes
    int conv_vec_ok, conv_ld_vec, copy_vec_ok, pool_vec_ok, elem_bytes;
    u64 *pool_box;       // [N*Ca*nslab] partial sums
    u64 *dk_box;         // [N*Ca*9]
    unsigned *err;       // raised when a bounded wait expires
    unsigned *epoch;     // [kGroups] call counters (kCtlStride words apart) = tag of the current call
    unsigned *done;      // [kGroups] blocks of the group that have announced their leave
    u64 *trace;          // development builds only
};

// Per-block state that item code touches.
struct Ctx {
    uint32_t tag;     // call tag, read lazily
    bool have_tag;
    bool last_item;   // the item being processed is the block's last
    bool announced;   // leave already announced
    unsigned left;    // thread kThreads-1 only: blocks of the group that had announced before this one
};

// Reads the call tag once per block, at a point where the caller's own loads are already
// in flight (it must not sit in front of them: results return in order).  A plain cached
// load: the value was written by the previous launch and only changes once this block's
// whole group has announced its leave.
__device__ __forceinline__ void need_tag(const FwdParams &p, Ctx &ctx)
{
    if (!ctx.have_tag) {
        ctx.tag = *(const volatile unsigned *)(p.epoch + (blockIdx.x % kGroups) * kCtlStride);
        ctx.have_tag = true;
    }
}

// Called once the loads of the block's last item are in flight: announce the leave, so the
// atomic's round trip is over long before the block ends.
__device__ __forceinline__ void announce_leave(const FwdParams &p, Ctx &ctx)
{
    if (ctx.last_item && !ctx.announced) {
        need_tag(p, ctx);
        // Every wavefront's copy of the tag must have arrived before the announcement can be
        // seen: once the whole group has announced, the group's counter advances.
        asm volatile("" ::"v"(ctx.tag) : "memory");
        __syncthreads();
        if (threadIdx.x == kThreads - 1)
            ctx.left = __hip_atomic_fetch_add(p.done + (blockIdx.x % kGroups) * kCtlStride, 1u,
                                              __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ctx.announced = true;
    }
}

// ---------------------------------------------------------------------------
// pool item (Eq. 4 line 2, first half).  Thread t adds elements
// base + (k*256 + t)*V + q for k, then q, ascending - the same order whether the
// 16-byte loads are usable or not - then a fixed tree over the block.  The
// decomposition depends on H*W only, so a batch reproduces its images run alone.
// ---------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void pool_item(const FwdParams &p, Ctx &ctx, unsigned item, float *s_red)
{
    constexpr int V = 16 / (int)sizeof(T);  // elements per 16-byte load
    constexpr int K = kPoolSlab / (kThreads * V);
    const int HW = p.H * p.W;
    const unsigned nc = fdiv(item, p.div_nslab);
    const int slab = (int)(item - nc * (unsigned)p.nslab);
    const unsigned n = fdiv(nc, p.div_ca);
    const unsigned c = nc - n * (unsigned)p.Ca;
    const T *plane = (const T *)p.x + ((size_t)n * p.C + c) * (size_t)HW;
    const int base = slab * kPoolSlab;
    float s = 0.f;
    if (p.pool_vec_ok && base + kPoolSlab <= HW) {
        u32x4 raw[K];
#pragma unroll
        for (int k = 0; k < K; ++k)
            raw[k] = *reinterpret_cast<const u32x4 *>(plane + base + (k * kThreads + (int)threadIdx.x) * V);
        need_tag(p, ctx);
        announce_leave(p, ctx);
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
        need_tag(p, ctx);
        announce_leave(p, ctx);
    }
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = s_red[0];
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) t += s_red[w];
        box_put(p.pool_box + item, t, ctx.tag);
    }
}

// ---------------------------------------------------------------------------
// The kernel estimator (Eq. 4 line 2, second half) of image n.  The GAP of a
// channel is finished in one fixed order everywhere: lane l of a wavefront adds
// slabs l, l+64, ... ascending, then the wavefront tree adds the lanes.  Then the
// estimator, one output per thread.  A gen item publishes all 9*C_a outputs; when
// an image has few slabs the conv items skip that hop and derive their own nine
// values with the same arithmetic.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float gelu_erf(float v)
{
    return 0.5f * v * (1.f + erff(v * 0.70710678118654752440f));
}

// bias + sum_k w[k] * in[k], accumulated in ascending k.  Weights are fetched eight at
// a time so their latencies overlap instead of adding up.
__device__ __forceinline__ float dot_row(const float *w, const float *in, int K, float bias)
{
    float s = bias;
    for (int k0 = 0; k0 < K; k0 += 8) {
        float wv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) wv[u] = k0 + u < K ? w[k0 + u] : 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (k0 + u < K) s = fmaf(wv[u], in[k0 + u], s);
    }
    return s;
}

// Whole block: waits for image n's pool mailboxes (staged through s_part), leaves the
// pooled means in s_g and (two-layer estimator) the hidden activations in s_t.  Ends
// with a barrier.
__device__ __forceinline__ void estimator_front(const FwdParams &p, uint32_t tag, unsigned n, float *s_part,
                                                float *s_g, float *s_t)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nslab = p.nslab, Ca = p.Ca;
    const u64 *img_boxes = p.pool_box + (size_t)n * Ca * nslab;
    if (nslab <= kStage) {
        const int G = kStage / nslab;  // whole channels per round
        for (int c0 = 0; c0 < Ca; c0 += G) {
            const int gc = Ca - c0 < G ? Ca - c0 : G;
            boxes_to_lds(img_boxes + (size_t)c0 * nslab, gc * nslab, s_part, tag, p.err);
            __syncthreads();
            for (int cg = wave; cg < gc; cg += kThreads / 64) {
                float s = 0.f;
                for (int k = lane; k < nslab; k += 64) s += s_part[cg * nslab + k];
                s = wave_sum(s);
                if (lane == 0) s_g[c0 + cg] = s / p.hw;
            }
            __syncthreads();
        }
    } else {
        // a channel has more slabs than fit: kStage at a time; kStage % 64 == 0 keeps every
        // slab on the lane its index selects
        for (int c = 0; c < Ca; ++c) {
            float s = 0.f;
            for (int k0 = 0; k0 < nslab; k0 += kStage) {
                const int cnt = nslab - k0 < kStage ? nslab - k0 : kStage;
                boxes_to_lds(img_boxes + (size_t)c * nslab + k0, cnt, s_part, tag, p.err);
                __syncthreads();
                if (wave == 0)
                    for (int k = lane; k < cnt; k += 64) s += s_part[k];
                __syncthreads();
            }
            if (wave == 0) {
                s = wave_sum(s);
                if (lane == 0) s_g[c] = s / p.hw;
            }
        }
        __syncthreads();
    }
    if (p.hidden > 0) {
        for (int m = threadIdx.x; m < p.hidden; m += kThreads)
            s_t[m] = gelu_erf(dot_row(p.w_down + (size_t)m * Ca, s_g, Ca, p.b_down ? p.b_down[m] : 0.f));
        __syncthreads();
    }
}

// One thread: estimator output o (= DK entry c*9 + i*3 + j) from what estimator_front left.
__device__ __forceinline__ float estimator_out(const FwdParams &p, int o, const float *s_g, const float *s_t)
{
    const float *in = p.hidden > 0 ? s_t : s_g;
    const int K = p.hidden > 0 ? p.hidden : p.Ca;
    return dot_row(p.w_up + (size_t)o * K, in, K, p.b_up ? p.b_up[o] : 0.f);
}

__device__ __forceinline__ void gen_item(const FwdParams &p, Ctx &ctx, unsigned n, float *s_part, float *s_g,
                                         float *s_t, u64 *rec)
{
    need_tag(p, ctx);
    announce_leave(p, ctx);
    estimator_front(p, ctx.tag, n, s_part, s_g, s_t);
    ESC_STAMP(rec, 3);
    for (int o = threadIdx.x; o < 9 * p.Ca; o += kThreads) {
        const float s = estimator_out(p, o, s_g, s_t);
        const size_t idx = (size_t)n * 9 * p.Ca + o;
        box_put(p.dk_box + idx, s, ctx.tag);
        if (p.dk_out) p.dk_out[idx] = s;
    }
}

// ---------------------------------------------------------------------------
// conv item (Eq. 4 line 3).  The zero-extended halo tile sits in LDS as fp32, and
// so do the channel's Ks x Ks weights.  Thread (tx, ty) produces outputs
// x = 4*tx..4*tx+3 of rows ty*RY..ty*RY+RY-1.  Each tile row segment it loads
// (KS+3 values, 16-byte reads) feeds up to RY kernel rows; a kernel row comes in
// with broadcast 16-byte reads.  DK's nine taps run afterwards from the same tile,
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
    static constexpr int WP = (KS + 3) & ~3;      // pitch of a weight row in LDS
    static constexpr int TILE_FLOATS = HR * PITCH;
    static constexpr int W_FLOATS = KS * WP;
};

template <int KS, int RY, typename T>
__device__ __forceinline__ void conv_item(const FwdParams &p, Ctx &ctx, unsigned item, float *tile, float *wl,
                                          float *s_dk, float *s_part, float *s_g, float *s_t, u64 *rec)
{
    using G = ConvGeom<KS, RY>;
    constexpr int PH = G::PH, OFF = G::OFF, TH = G::TH, HR = G::HR, HC = G::HC, PITCH = G::PITCH,
                  NV = G::NV, WP = G::WP;
    const int H = p.H, W = p.W;

    const unsigned b1 = fdiv(item, p.div_tiles_x);
    const int txi = (int)(item - b1 * p.div_tiles_x.d);
    const unsigned nc = fdiv(b1, p.div_tiles_y);
    const int tyi = (int)(b1 - nc * p.div_tiles_y.d);
    const unsigned n = fdiv(nc, p.div_ca);
    const int c = (int)(nc - n * (unsigned)p.Ca);
    const size_t plane_off = ((size_t)n * p.C + c) * (size_t)H * (size_t)W;
    const T *xp = (const T *)p.x + plane_off;
    T *op = (T *)p.out + plane_off;
    const int x0 = txi * kTileW, y0 = tyi * TH;

    // this channel's weights, fetched together with the tile
    constexpr int KW = (KS * KS + kThreads - 1) / kThreads;
    const float *lkc = p.lk + (size_t)c * p.lk_cstride;
    float wreg[KW];
#pragma unroll
    for (int m = 0; m < KW; ++m) {
        const int idx = m * kThreads + (int)threadIdx.x;
        wreg[m] = idx < KS * KS ? lkc[idx] : 0.f;
    }

    // halo tile -> LDS, zero outside the image
    if (p.conv_ld_vec) {
        // W % 4 == 0 and an aligned base: fetch whole 4-element chunks aligned in global
        // memory (each lies entirely inside or outside the image), all loads in flight
        // before the first LDS write.  A chunk lands at LDS column 4j - A.
        constexpr int A = (4 - PH % 4) % 4;
        constexpr int NCH = (HC + A + 3) / 4;
        constexpr int TOT = HR * NCH;
        constexpr int K = (TOT + kThreads - 1) / kThreads;
        const int g0 = x0 - PH - A;
        float v[K][4];
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const int q = k * kThreads + (int)threadIdx.x;
            const int r = q / NCH, j = q - r * NCH;
            const int gy = y0 - PH + r, gx = g0 + 4 * j;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[k][e] = 0.f;
            if (q < TOT && gy >= 0 && gy < H && gx >= 0 && gx < W) load4(xp + (size_t)gy * W + gx, v[k]);
        }
        if (p.dk_mode >= kDkBoxes) need_tag(p, ctx);
        announce_leave(p, ctx);
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const int q = k * kThreads + (int)threadIdx.x;
            const int r = q / NCH, j = q - r * NCH;
            if (q < TOT) {
                float *dst = tile + r * PITCH + 4 * j - A;
                if (A == 0) {
                    *reinterpret_cast<float4 *>(dst) = make_float4(v[k][0], v[k][1], v[k][2], v[k][3]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int cc = 4 * j - A + e;
                        if (cc >= 0 && cc < HC) dst[e] = v[k][e];
                    }
                }
            }
        }
    } else {
        for (int idx = threadIdx.x; idx < HR * HC; idx += kThreads) {
            const int r = idx / HC, cc = idx - r * HC;
            const int gy = y0 - PH + r, gx = x0 - PH + cc;
            float v = 0.f;
            if (gy >= 0 && gy < H && gx >= 0 && gx < W) v = to_f32(xp[(size_t)gy * W + gx]);
            tile[r * PITCH + cc] = v;
        }
        if (p.dk_mode >= kDkBoxes) need_tag(p, ctx);
        announce_leave(p, ctx);
    }
#pragma unroll
    for (int m = 0; m < KW; ++m) {
        const int idx = m * kThreads + (int)threadIdx.x;
        if (idx < KS * KS) wl[(idx / KS) * WP + idx % KS] = wreg[m];
    }
    __syncthreads();
    ESC_STAMP(rec, 3);

    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float acc[RY][4];
#pragma unroll
    for (int oy = 0; oy < RY; ++oy)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[oy][q] = 0.f;

    const float *trow = tile + (ty * RY) * PITCH + 4 * tx;

#pragma unroll 1
    for (int r = 0; r < RY + KS - 1; ++r) {
        float v[NV];
        if (OFF == 0) {
            const float4 *src = reinterpret_cast<const float4 *>(trow + r * PITCH);
#pragma unroll
            for (int k = 0; k < NV / 4; ++k) {
                const float4 f = src[k];
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
                float w[WP];
                const float4 *wsrc = reinterpret_cast<const float4 *>(wl + i * WP);
#pragma unroll
                for (int k = 0; k < WP / 4; ++k) {
                    const float4 f = wsrc[k];
                    w[4 * k + 0] = f.x;
                    w[4 * k + 1] = f.y;
                    w[4 * k + 2] = f.z;
                    w[4 * k + 3] = f.w;
                }
#pragma unroll
                for (int j = 0; j < KS; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) acc[oy][q] = fmaf(w[j], v[j + q], acc[oy][q]);
            }
        }
    }
#ifdef ESC_TRACE
#pragma unroll
    for (int oy = 0; oy < RY; ++oy)
#pragma unroll
        for (int q = 0; q < 4; ++q) asm volatile("" ::"v"(acc[oy][q]));
#endif
    ESC_STAMP(rec, 4);

    if (p.dk_mode != kDkNone) {
        const size_t dk_idx = ((size_t)n * p.Ca + c) * 9;
        if (p.dk_mode == kDkDirect) estimator_front(p, ctx.tag, n, s_part, s_g, s_t);
        ESC_STAMP(rec, 12);
        if (threadIdx.x < 9) {
            float d;
            if (p.dk_mode == kDkDirect)
                d = estimator_out(p, c * 9 + (int)threadIdx.x, s_g, s_t);
            else if (p.dk_mode == kDkBoxes)
                d = box_get(p.dk_box + dk_idx + threadIdx.x, ctx.tag, p.err);
            else
                d = p.dk_in[dk_idx + threadIdx.x];
            s_dk[threadIdx.x] = d;
        }
        __syncthreads();
        ESC_STAMP(rec, 5);
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
__device__ __forceinline__ void copy_item(const FwdParams &p, Ctx &ctx, unsigned item)
{
    const unsigned n = fdiv(item, p.div_chunks);
    const size_t chunk = (size_t)(item - n * p.div_chunks.d);
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
        announce_leave(p, ctx);
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
        announce_leave(p, ctx);
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
__global__ __launch_bounds__(kThreads, kBlocksPerCu) void forward_kernel(const FwdParams p)
{
    using G = ConvGeom<(KS > 0 ? KS : 1), RY>;
    __shared__ __align__(16) float tile[KS > 0 ? G::TILE_FLOATS : 4];
    __shared__ __align__(16) float wl[KS > 0 ? G::W_FLOATS : 4];
    __shared__ float s_part[kStage];
    __shared__ float s_g[kMaxCa];
    __shared__ float s_t[kMaxHidden];
    __shared__ float s_small[16];

    const unsigned first_mixed = p.n_pool + p.n_gen;
    const unsigned total = first_mixed + p.n_conv + p.n_copy;
    Ctx ctx;
    ctx.tag = 0;
    ctx.have_tag = false;
    ctx.last_item = false;
    ctx.announced = false;
    ctx.left = 0;
    for (unsigned item = blockIdx.x; item < total; item += gridDim.x) {
        u64 *rec = nullptr;
#ifdef ESC_TRACE
        if (p.trace != nullptr) {
            rec = p.trace + (size_t)item * 16;
            if (threadIdx.x == 0) {
                rec[0] = item;
                rec[1] = ((u64)__builtin_amdgcn_s_getreg((31 << 11) | 4) << 32) | blockIdx.x;
                rec[15] = __builtin_amdgcn_s_getreg((31 << 11) | 20);
                rec[13] = clock64();
            }
        }
#endif
        ESC_STAMP(rec, 2);
        ctx.last_item = item + gridDim.x >= total;
        if (item < p.n_pool) {
            pool_item<T>(p, ctx, item, s_small);
        } else if (item < first_mixed) {
            gen_item(p, ctx, item - p.n_pool, s_part, s_g, s_t, rec);
        } else {
            const unsigned j = item - first_mixed;
            const unsigned group = p.mix_a + p.mix_b;
            bool is_conv;
            unsigned idx;
            if (j < p.mix_groups * group) {
                const unsigned g = fdiv(j, p.div_mix), r = j - g * group;
                is_conv = r < p.mix_a;
                idx = is_conv ? g * p.mix_a + r : g * p.mix_b + (r - p.mix_a);
            } else {
                const unsigned jj = j - p.mix_groups * group;
                const unsigned conv_left = p.n_conv - p.mix_groups * p.mix_a;
                is_conv = jj < conv_left;
                idx = is_conv ? p.mix_groups * p.mix_a + jj : p.mix_groups * p.mix_b + (jj - conv_left);
            }
            if (is_conv) {
                if constexpr (KS > 0) conv_item<KS, RY, T>(p, ctx, idx, tile, wl, s_small, s_part, s_g, s_t, rec);
            } else {
                copy_item(p, ctx, idx);
            }
        }
        ESC_STAMP(rec, 6);
#ifdef ESC_TRACE
        if (rec != nullptr && threadIdx.x == 0) rec[14] = clock64();
#endif
        __syncthreads();  // LDS is reused by the next item
    }
    // A block without items still belongs to its group.  The last block of a group to have
    // announced its leave opens the next call for the group: leave counter back to zero, tag + 1.
    ctx.last_item = true;
    announce_leave(p, ctx);
    if (threadIdx.x == kThreads - 1) {
        const unsigned g = blockIdx.x % kGroups;
        const unsigned members = (gridDim.x - g + kGroups - 1) / kGroups;
        if (ctx.left == members - 1) {
            __hip_atomic_store(p.done + g * kCtlStride, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(p.epoch + g * kCtlStride, ctx.tag + 1u == 0u ? 1u : ctx.tag + 1u, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// Control block at the start of the workspace, in 32-bit words: word 0 the error word, then
// from kCtlEpochWord one call counter per group and from kCtlDoneWord one leave counter per
// group, each kCtlStride words apart.  Preparation: everything zero, call counters 1 (tag 0
// is what empty mailboxes carry).
constexpr size_t kCtlErrWord = 0;
constexpr size_t kCtlEpochWord = kCtlStride;
constexpr size_t kCtlDoneWord = kCtlEpochWord + (size_t)kGroups * kCtlStride;
constexpr size_t kCtlWords = kCtlDoneWord + (size_t)kGroups * kCtlStride;

__global__ void ws_init_kernel(uint32_t *ptr, size_t words)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const bool is_epoch = i >= kCtlEpochWord && i < kCtlDoneWord && (i - kCtlEpochWord) % kCtlStride == 0;
    if (i < words) ptr[i] = is_epoch ? 1u : 0u;
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
    l->ctl_off = off;
    off = round_up(off + kCtlWords * sizeof(uint32_t), kWsAlign);
    l->pool_off = off;
    off = round_up(off + (size_t)N * Ca * l->nslab * sizeof(u64), kWsAlign);
    l->dk_off = off;
    off = round_up(off + (size_t)N * Ca * 9 * sizeof(u64), kWsAlign);
    l->total = off;
    return true;
}

FastDiv make_div(uint32_t d)
{
    FastDiv f;
    if (d == 0) d = 1;
    uint32_t l = 0;
    while (((uint64_t)1 << l) < d) ++l;
    f.d = d;
    f.mul = (uint32_t)((((uint64_t)1 << 32) * (((uint64_t)1 << l) - d)) / d + 1);
    f.shift = l;
    return f;
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
    if (need < kCtlWords * sizeof(uint32_t)) need = kCtlWords * sizeof(uint32_t);
    if (ws == nullptr || ((uintptr_t)ws % kWsAlign) != 0 || ws_bytes < need) return ESC_ERR_WORKSPACE;
    return ESC_OK;
}

#ifdef ESC_TRACE
u64 *g_trace = nullptr;
#endif

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

// conv and copy items alternate in small groups so that both kinds are in flight together
void set_mix(FwdParams &p)
{
    unsigned a = 1, b = 1;
    if (p.n_conv > 0 && p.n_copy > 0) {
        if (p.n_conv >= p.n_copy) {
            a = (p.n_conv + p.n_copy / 2) / p.n_copy;
            if (a > 16) a = 16;
        } else {
            b = (p.n_copy + p.n_conv / 2) / p.n_conv;
            if (b > 16) b = 16;
        }
        const unsigned ga = p.n_conv / a, gb = p.n_copy / b;
        p.mix_groups = ga < gb ? ga : gb;
    } else {
        p.mix_groups = 0;
    }
    p.mix_a = a;
    p.mix_b = b;
    p.div_mix = make_div(a + b);
}

template <int KS, int RY, typename T>
esc_status launch_variant(FwdParams &p, hipStream_t s)
{
    // the kernel is compiled for kBlocksPerCu resident blocks per compute unit (register
    // budget via __launch_bounds__, LDS <= 40 KiB of 160 KiB), so this grid is co-resident
    const int cus = device_cus();
    if (cus < 1) return ESC_ERR_HIP;
    const u64 total = (u64)p.n_pool + p.n_gen + p.n_conv + p.n_copy;
    if (total == 0) return ESC_OK;
    if (total >= ((u64)1 << 30)) return ESC_ERR_UNSUPPORTED;  // item + grid must not wrap
    set_mix(p);
    const u64 cap = (u64)kBlocksPerCu * (u64)cus;
    unsigned grid = (unsigned)(total < cap ? total : cap);
    if (grid < (unsigned)kGroups) grid = kGroups;  // every group of blocks needs a member
    // a block's items are grid apart: keep that stride coprime with the conv/copy pattern
    const unsigned pattern = p.mix_a + p.mix_b;
    auto gcd = [](unsigned a, unsigned b) {
        while (b) {
            const unsigned t = a % b;
            a = b;
            b = t;
        }
        return a;
    };
    while (total > grid && grid > (unsigned)kGroups && gcd(grid, pattern) != 1) --grid;
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
        const int tiles_x = (p.W + kTileW - 1) / kTileW;
        const int tiles_y = (p.H + th - 1) / th;
        p.div_tiles_x = make_div((uint32_t)tiles_x);
        p.div_tiles_y = make_div((uint32_t)tiles_y);
        const size_t n_conv = (size_t)tiles_x * tiles_y * p.N * p.Ca;
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
    p.div_nslab = make_div((uint32_t)l.nslab);
    p.div_ca = make_div((uint32_t)(Ca > 0 ? Ca : 1));
    p.div_tiles_x = p.div_tiles_y = p.div_chunks = p.div_mix = make_div(1);
    if (gen != nullptr && Ca > 0) {
        p.dk_mode = ((size_t)Ca * l.nslab <= (size_t)kDirectMaxBoxes) ? kDkDirect : kDkBoxes;
        p.hidden = gen->hidden;
        p.w_down = gen->w_down;
        p.b_down = gen->b_down;
        p.w_up = gen->w_up;
        p.b_up = gen->b_up;
        const size_t n_pool = (size_t)N * Ca * l.nslab;
        if (n_pool >= ((size_t)1 << 30)) return ESC_ERR_UNSUPPORTED;
        p.n_pool = (unsigned)n_pool;
        p.n_gen = p.dk_mode == kDkBoxes ? (unsigned)N : 0u;
        const size_t plane_bytes = (size_t)H * W * p.elem_bytes;
        p.pool_vec_ok = ((uintptr_t)x % 16 == 0) && (plane_bytes % 16 == 0);
    }
    char *w = (char *)workspace;
    p.err = (unsigned *)(w + l.ctl_off) + kCtlErrWord;
    p.epoch = (unsigned *)(w + l.ctl_off) + kCtlEpochWord;
    p.done = (unsigned *)(w + l.ctl_off) + kCtlDoneWord;
#ifdef ESC_TRACE
    p.trace = g_trace;
#endif
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
    hipLaunchKernelGGL(ws_init_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream,
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
    if (hipMemcpyAsync(&v, (const uint32_t *)workspace + kCtlErrWord, sizeof v, hipMemcpyDeviceToHost,
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
    p.dk_mode = kDkBoxes;  // no conv items here: gen items write dk_out
    p.n_gen = (unsigned)N;
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
    if (p.dk_in != nullptr) p.dk_mode = kDkGiven;
    // aligned 4-element chunk loads of the halo tile need W % 4 == 0 and an aligned base
    p.conv_ld_vec = (W % 4 == 0) && (xa % (4 * es) == 0);
    // 16-byte (fp32) / 8-byte (bf16) row stores need W % 4 == 0 and an aligned base
    p.conv_vec_ok = (W % 4 == 0) && (oa % (4 * es) == 0);
    if (C_a < C) {
        const size_t plane = (size_t)H * W * es;
        p.img_bytes = plane * C;
        p.idt_off = plane * C_a;
        p.idt_len = plane * (C - C_a);
        const size_t chunks = (p.idt_len + kCopyChunk - 1) / kCopyChunk;
        if (chunks * (size_t)N >= ((size_t)1 << 30)) return ESC_ERR_UNSUPPORTED;
        p.div_chunks = make_div((uint32_t)chunks);
        p.n_copy = (unsigned)(chunks * N);
        p.copy_vec_ok = (xa % 16 == 0) && (oa % 16 == 0) && (p.img_bytes % 16 == 0) && (p.idt_off % 16 == 0);
    }
    const int ks_variant = C_a > 0 ? Ks : 0;
    return dt == ESC_F32 ? launch_typed<float>(p, ks_variant, (hipStream_t)stream)
                         : launch_typed<bf16_t>(p, ks_variant, (hipStream_t)stream);
}

#ifdef ESC_TRACE
void esc_debug_set_trace(void *buf) { g_trace = (u64 *)buf; }
#endif

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

// Device code of the ConvAttn forward for gfx950 (MI355X): the work items and the one
// persistent kernel that runs them.  Included by esc_variants.hip (which instantiates the
// kernel for one kernel size per translation unit) and by esc_api.hip (host side, C ABI).
//
// The operation is Eq. 4 of the ESC paper with the depth-wise large kernel of
// the paragraph around Eq. 5.  With fp32 storage everything is plain fp32 vector
// arithmetic (a depth-wise convolution has no reduction shared between outputs); with
// bf16 storage and Ks <= 17 the tap loop multiplies bf16 tile rows with the kernel rows'
// Toeplitz matrices on the matrix cores, fp32 accumulation (MatrixGeom).
//
// One launch does the whole forward.  The work is cut into items, in this order in
// every die's list:
//
//   pool items   GAP partial sums of the attention slice, four 64 x 32 pixel tiles each;
//                left out when every conv item is resident at once - then each conv
//                item publishes the sums of its own tile from LDS ("fused pooling")
//   gen items    one per image with few pool tiles: finish the GAP, run the kernel
//                estimator, publish DK (esc_dynkernel_gen: also write it out)
//   gsum items   for images with many pool tiles: one per (image, channel), publish the
//                channel's mean; one gen item per image behind them turns the means into DK
//   conv items   one 64 x (16*RY) output tile of one (image, channel) plane: LK taps
//                from an LDS halo tile with the channel's weights staged in LDS, then
//                DK's nine taps once DK is known (asked for from inside the tap loop)
//   copy items   a chunk of the identity channels, interleaved with the conv items so
//                streaming and arithmetic overlap on every compute unit
//
// Every die of the chip gets a contiguous eighth of each kind of item.  A call that fits
// in one round of resident blocks is dealt statically; a longer one deals each die's list
// to its eight block groups, whose blocks take entry after entry from a queue counter.
// An item only ever waits for items that are earlier in the lists or dealt in the first
// round, a waiting block holds no reservation on later entries, and pool items wait for
// nothing and come first, so every wait ends as long as the blocks of the grid are
// co-resident (the host sizes the grid to what the kernel is compiled to fit) - and each
// wait is bounded anyway: on expiry the block raises the error word of the workspace and
// goes on.
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
// Facts about the machine that shape the code (measured, not assumed):
//   - an FMA whose multiplier sits in a scalar register issues at about 0.27 per clock
//     and SIMD, one with both operands in vector registers at up to 0.375 (four
//     wavefronts; 0.34 with two, 0.20 with one), so the tap weights are read from LDS
//     (a broadcast read) into vector registers; the bf16 dot instruction saturates at
//     0.236, so two taps per instruction gain little on a full compute unit - the bf16
//     tap loop therefore runs on the matrix cores;
//   - vector-memory results return in order, so an atomic with a slow answer delays
//     every later load of its wavefront, and a wait for a load is also a wait for every
//     store issued before it: the leave announcement is issued where no wait on memory
//     follows soon and no mailbox store precedes (for conv items: behind the barrier
//     that ends the tile fill);
//   - a mailbox hop takes 0.4 us on an idle chip and about 2 us beside streaming
//     traffic, whichever dies the two blocks are on;
//   - a thousand atomics on one address take tens of microseconds: nothing here
//     has more than a handful of blocks on the same word;
//   - a load behind a condition lands in a basic block of its own and the compiler then
//     waits for it before issuing the next: loads that should overlap are unconditional
//     (clamped addresses, results masked afterwards);
//   - any private-segment (scratch) use costs a launch a fixed microsecond or more, and the
//     compiler spills as soon as thread-index arithmetic is hoisted out of the item loop
//     and held through every item: each phase takes the thread index afresh (opaque_tid).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "esc_convattn.h"
#include "esc_dense_weights.hpp"

namespace esc {

constexpr int kThreads = 256;      // 4 wavefronts per block
constexpr int kTileW = 64;         // conv tile width: 16 lanes x 4 outputs
constexpr int kMaxCa = 256;
constexpr int kMaxHidden = 256;
constexpr int kMaxKs = 31;
constexpr size_t kWsAlign = 256;
constexpr unsigned kSpinLimit = 1u << 20;  // bounded wait: about a second, far beyond any real wait
constexpr int kBlocksPerCu = 4;    // resident blocks per compute unit the kernel is compiled for (<= 128 VGPRs)
constexpr int kCopyVecPerThread = 4;
constexpr size_t kCopyPiece = (size_t)kThreads * 16 * kCopyVecPerThread;  // bytes a block has in flight
constexpr size_t kGrain = (size_t)kThreads * 16;  // a grain of the carried copy: 16 bytes per thread of a conv item
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
// Which conv variants move a share of the pass-through copy from inside their tap loops
// (carried copy): the four-row blocks with bf16 storage.  Their calls fill every block
// slot with conv items, so the streaming finds no block to run in beside them, and idle
// memory pipes under their tap loops.
// Measured, the other variants lose by it: short fp32 calls last as long as their chain of
// tile load, taps, estimator and store, which extra traffic stretches, and long fp32 calls
// already alternate conv and copy items.
constexpr bool conv_carries(int ks, int ry, bool bf16) { return bf16 && ry == 4 && ks <= 17; }
// grains (16 bytes per thread, 4 KiB per block) such an item has room for in its registers
constexpr int kCarryGrains = 6;
constexpr int conv_carry_grains(int ks, int ry, bool bf16) { return conv_carries(ks, ry, bf16) ? kCarryGrains : 0; }
typedef __amdgpu_buffer_rsrc_t CarryRsrc;
constexpr int kRawBufferFlags = 0x00020000;  // raw buffer (no stride, no swizzle), 32-bit data format
constexpr int kBufferNt = 2;                 // non-temporal

struct FastDiv {
    uint32_t d, mul, shift;
};

// ---------------------------------------------------------------------------
// kernel arguments
// ---------------------------------------------------------------------------
enum : int {
    kDkNone = 0,    // DK = 0
    kDkGiven = 1,   // caller's dk_in
    kDkBoxes = 2,   // published by a gen item (esc_dynkernel_gen: the gen items also write dk_out)
    kDkDirect = 3,  // each conv item finishes the GAP and runs its nine estimator outputs itself
    kDkFromG = 4,   // host only, while a call is set up: larger planes, whose means come from gsum
                    // items (n_gsum > 0); the call then runs as kDkBoxes or kDkMeans
    kDkMeans = 5    // larger planes, small estimator: each conv item collects its image's channel
                    // means from the gsum items' mailboxes and runs its nine estimator outputs itself
                    // (one mailbox hop fewer than through a gen item)
};
enum : int {
    kPoolNone = 0,   // no estimator in this call
    kPoolItems = 1,  // pool items read the attention slice and publish the partial sums
    kPoolFused = 2   // every conv item is resident at once: each publishes the sum of its own tile
};
// an image with at most this many pool mailboxes (C_a * pool tiles) has them read in one
// round by whoever finishes its GAP (a gen item, or each conv item); larger ones go
// through channel-mean items
constexpr int kDirectMaxBoxes = 512;
constexpr int kPoolTileW = 64, kPoolTileH = 32;  // the GAP is cut into 64 x 32 pixel tiles
constexpr int kPoolBatch = 4;                    // pool tiles per pool item

struct FwdParams {
    const void *x;
    void *out;
    const float *lk;
    long lk_cstride;
    const float *dk_in;  // DK given by the caller (no estimator), or NULL
    float *dk_out;       // esc_dynkernel_gen: where the estimator's DK goes, else NULL
    const float *out_add;  // [N*Ca] a constant per (image, channel) added to every output of its plane before the
                           // store's rounding (the backward's GAP term), or NULL
    const float *w_down, *b_down, *w_up, *b_up;
    int hidden;
    int dk_mode;         // where conv items take DK from (kDk*)
    int pool_mode;       // who computes the GAP partial sums (kPool*)
    int N, C, Ca, H, W;
    int out_c;           // channels per image of `out` (C; C_a when only F_res is written)
    int ptiles_x, ptiles;  // pool tiles per row of tiles / per (image, channel) plane
    float hw;            // H*W as a float, the GAP divisor
    unsigned n_pool, n_gen, n_conv, n_copy;  // item counts
    unsigned n_pool_tiles;                   // N * C_a * ptiles (a pool item covers kPoolBatch of them)
    // conv and copy items alternate in groups of mix_a conv + mix_b copy items while both
    // last; the rest of the conv items follow, then the rest of the copy items
    unsigned mix_a, mix_b;
    FastDiv div_ptiles, div_ptiles_x, div_ca, div_tiles_x, div_tiles_y, div_chunks, div_mix, div_mix_a, div_mix_b;
    size_t img_bytes, idt_off, idt_len;      // pass-through range of one image, in bytes
    size_t copy_chunk;                       // bytes per copy item (a multiple of kCopyPiece)
    int conv_vec_ok, conv_ld_vec, copy_vec_ok, elem_bytes;
    u64 *pool_box;       // [N*Ca*ptiles] partial sums
    u64 *dk_box;         // [N*Ca*9]
    u64 *g_box;          // [N*Ca] channel means (calls with gsum items)
    unsigned n_gsum;     // channel-mean calls: the first n_gsum gen entries are gsum items, one per
                         // (image, channel); the N gen items behind them turn the means into DK
    unsigned *err;       // raised when a bounded wait expires
    unsigned *epoch;     // [kGroups] call counters (kCtlStride words apart) = tag of the current call
    unsigned *done;      // [kGroups] blocks of the group that have announced their leave
    unsigned *queue;     // [kGroups] entries of the group's list handed out beyond the first per block
    int dynamic;         // blocks take their further entries from the group's queue
    int staged;          // host only: launch the kernel flavour with the staged estimator items (and out_add)
    // Every conv item is resident from the start (fused pooling) and the call is so short
    // that the conv items' chain of load, taps, estimator and store is what it lasts: the
    // copy items then keep little in flight, so that the conv items' few accesses (tile,
    // mailboxes) come back quickly; measured, a full-rate copy beside them costs more than
    // it saves.
    int copy_gentle;
    // The variant without conv items only (the estimator launch of a dense call): its copy
    // entries are not copy items but pieces of 256 entries of the dense kernel's A-operand
    // table, built from aux_lk beside the pooling (aux_n entries; 0 = none).
    const float *aux_lk;
    uint32_t *aux_wa;
    int aux_n, aux_Ca, aux_Ks, aux_Kse, aux_nw;
    // Carried copy: conv item j of an image (j counts its tiles channel-major) moves bytes
    // [j * carry_g * kGrain, (j + 1) * carry_g * kGrain) of the image's pass-through range
    // (loaded behind its tile, stored behind its tap loop); the copy items cover what lies
    // beyond copy_off (bytes from the start of the range).  0 = nothing is carried.
    unsigned carry_g;
    size_t copy_off;
};

// The kernel's parameter block as the item functions see it: a pointer into the kernel
// argument segment (constant address space), read with scalar loads where needed instead
// of being held in registers across a whole item.
typedef const __attribute__((address_space(4))) FwdParams *ParamsPtr;

constexpr unsigned kXcds = 8;
constexpr int kPrioHigh = 3;  // wavefront priority outside the tap loop

// Control block at the start of the workspace, in 32-bit words: word 0 the error word, then
// from kCtlEpochWord one call counter per group, from kCtlDoneWord one leave counter per
// group and from kCtlQueueWord one queue counter per group, each kCtlStride words apart.
// Preparation: everything zero, call counters 1 (tag 0 is what empty mailboxes carry).
constexpr size_t kCtlErrWord = 0;
constexpr size_t kCtlEpochWord = kCtlStride;
constexpr size_t kCtlDoneWord = kCtlEpochWord + (size_t)kGroups * kCtlStride;
constexpr size_t kCtlQueueWord = kCtlDoneWord + (size_t)kGroups * kCtlStride;
constexpr size_t kCtlWords = kCtlQueueWord + (size_t)kGroups * kCtlStride;


}  // namespace esc

namespace esc {
namespace {

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

// two results rounded to nearest even and packed, a in the low half: the hardware's packed
// conversion (v_cvt_pk_bf16_f32), one instruction where the shifts and adds above are a dozen
__device__ __forceinline__ uint32_t f32_pack2_bf16(float a, float b)
{
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
}

__device__ __forceinline__ void store1(float *p, float v) { *p = v; }
__device__ __forceinline__ void store1(bf16_t *p, float v) { p->bits = f32_to_bf16_bits(v); }

// Output stores are non-temporal: nothing in the call reads them back, and lines that do
// not linger in the L2 shorten the write-back at the end of the kernel (measured).
__device__ __forceinline__ void store4(float *p, const float *v)
{
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const f32x4 t = {v[0], v[1], v[2], v[3]};
    __builtin_nontemporal_store(t, reinterpret_cast<f32x4 *>(p));
}
__device__ __forceinline__ void store4(bf16_t *p, const float *v)
{
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    u32x2 w;
    w.x = f32_pack2_bf16(v[0], v[1]);
    w.y = f32_pack2_bf16(v[2], v[3]);
    __builtin_nontemporal_store(w, reinterpret_cast<u32x2 *>(p));
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

// the same four bf16 elements, left as they are (two per 32-bit word, lower address low)
__device__ __forceinline__ uint2 load4_raw(const bf16_t *p) { return *reinterpret_cast<const uint2 *>(p); }
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// x / d for x < 2^31 by multiply-high and shift (host fills mul and shift)
__device__ __forceinline__ uint32_t fdiv(uint32_t x, uint32_t mul, uint32_t shift)
{
    return (__umulhi(x, mul) + x) >> shift;
}

// Values hidden from the optimiser: what is computed from them cannot be moved above the
// point where they are made, which keeps a later phase's addresses out of the registers of
// an earlier one.
__device__ __forceinline__ unsigned opaque_u(unsigned v)
{
    asm volatile("" : "+s"(v));
    return v;
}
__device__ __forceinline__ int opaque_tid()
{
    int t = (int)threadIdx.x;
    asm volatile("" : "+v"(t));
    return t;
}

// ---------------------------------------------------------------------------
// mailboxes
// ---------------------------------------------------------------------------
__device__ __forceinline__ void box_put(u64 *box, float v, uint32_t tag)
{
    __hip_atomic_store(box, ((u64)tag << 32) | (u64)__float_as_uint(v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}

// Waits (bounded) until the mailbox carries this call's tag.  On expiry raises *err and
// hands back NaN, so that whatever is computed from the missing value shows in the output.
__device__ __forceinline__ float box_get(const u64 *box, uint32_t tag, unsigned *err)
{
    for (unsigned spin = 0; spin < kSpinLimit; ++spin) {
        const u64 v = __hip_atomic_load(box, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((uint32_t)(v >> 32) == tag) return __uint_as_float((uint32_t)v);
        __builtin_amdgcn_s_sleep(2);
    }
    __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return __uint_as_float(0x7fc00000u);
}

// Whole block: waits (bounded) for cnt (<= PER * kPollThreads) consecutive mailboxes and
// copies their values to dst[0..cnt).  A thread's polls are issued together so their round trips overlap.
// With `have_first` the caller has already issued the first round into v.
template <int PER>
__device__ __forceinline__ void boxes_to_lds(const u64 *boxes, int cnt, float *dst, uint32_t tag, unsigned *err,
                                             u64 (&v)[PER], bool have_first)
{
    const int tid = opaque_tid();
    bool pend[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) pend[u] = tid < kPollThreads && tid + u * kPollThreads < cnt;
    bool any = false;
    for (unsigned spin = 0; spin < kSpinLimit; ++spin) {
        if (spin > 0 || !have_first) {
#pragma unroll
            for (int u = 0; u < PER; ++u)
                if (pend[u])
                    v[u] = __hip_atomic_load(boxes + tid + u * kPollThreads, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
        }
        any = false;
#pragma unroll
        for (int u = 0; u < PER; ++u)
            if (pend[u]) {
                if ((uint32_t)(v[u] >> 32) == tag) {
                    dst[tid + u * kPollThreads] = __uint_as_float((uint32_t)v[u]);
                    pend[u] = false;
                } else {
                    any = true;
                }
            }
        if (!any) break;
        __builtin_amdgcn_s_sleep(2);
    }
    if (any) {  // expired: raise the error word; the values that never came read as NaN
        __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int u = 0; u < PER; ++u)
            if (pend[u]) dst[tid + u * kPollThreads] = __uint_as_float(0x7fc00000u);
    }
}

// Sum over the 64 lanes of a wavefront, returned in every lane.  Data-parallel-primitive
// moves inside the vector ALU (a handful of cycles each; the LDS-crossbar shuffles they
// replace cost over a hundred): an inclusive scan inside each row of 16 lanes, then the
// row totals are carried over with the two row-broadcast steps; lane 63 ends with the
// total.  The order of the additions is fixed, which is all the callers rely on.
__device__ __forceinline__ float wave_sum(float v)
{
    constexpr int kRowShr = 0x110, kRowBcast15 = 0x142, kRowBcast31 = 0x143;
    auto dpp = [](float x, auto ctrl, auto row_mask) {
        return __builtin_bit_cast(
            float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value,
                                               decltype(row_mask)::value, 0xf, false));
    };
    v += dpp(v, std::integral_constant<int, kRowShr + 1>{}, std::integral_constant<int, 0xf>{});
    v += dpp(v, std::integral_constant<int, kRowShr + 2>{}, std::integral_constant<int, 0xf>{});
    v += dpp(v, std::integral_constant<int, kRowShr + 4>{}, std::integral_constant<int, 0xf>{});
    v += dpp(v, std::integral_constant<int, kRowShr + 8>{}, std::integral_constant<int, 0xf>{});
    v += dpp(v, std::integral_constant<int, kRowBcast15>{}, std::integral_constant<int, 0xa>{});
    v += dpp(v, std::integral_constant<int, kRowBcast31>{}, std::integral_constant<int, 0xc>{});
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// Running sum along each row of 16 lanes (lane 15 of a row ends with the row's total).
__device__ __forceinline__ float row_sum(float v)
{
    constexpr int kRowShr = 0x110;
    auto dpp = [](float x, auto ctrl) {
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x),
                                                                     decltype(ctrl)::value, 0xf, 0xf, false));
    };
    v += dpp(v, std::integral_constant<int, kRowShr + 1>{});
    v += dpp(v, std::integral_constant<int, kRowShr + 2>{});
    v += dpp(v, std::integral_constant<int, kRowShr + 4>{});
    v += dpp(v, std::integral_constant<int, kRowShr + 8>{});
    return v;
}

// die `die`'s contiguous share of n items: [base, base + cnt)
__device__ __forceinline__ void die_share(unsigned n, unsigned die, unsigned &base, unsigned &cnt)
{
    const unsigned q = n / kXcds, r = n % kXcds;
    cnt = q + (die < r ? 1u : 0u);
    base = die * q + (die < r ? die : r);
}

// LDS of a block, shared by all item kinds: the conv tile and weights are sized for the
// largest variant (Ks = 17 with 4-row register blocks; Ks = 31 with 2-row blocks).
constexpr int kLdsTileFloats = 6400;
constexpr int kLdsWeightFloats = 31 * 32;
__shared__ __align__(16) float g_tile[kLdsTileFloats];
__shared__ __align__(16) float g_wl[kLdsWeightFloats];
__shared__ float g_part[kStage];
__shared__ __align__(16) float g_g[kMaxCa];
__shared__ __align__(16) float g_t[kMaxHidden];
__shared__ float g_small[16];
__shared__ float g_red[4 * kPoolBatch];  // wavefront totals of the pool tiles being finished
__shared__ unsigned g_next[2];

// Per-block state that item code touches.
struct Ctx {
    uint32_t tag;     // call tag, read lazily
    bool have_tag;
    bool last_item;   // the item being processed is the block's last
    bool announced;   // leave already announced
    unsigned left;    // thread kThreads-1 only: blocks of the group that had announced before this one
    unsigned claim;   // thread kThreads-1 only: what the group's queue returned for the block's next entry
};

// Reads the call tag once per block, at a point where the caller's own loads are already
// in flight (it must not sit in front of them: results return in order).  A plain cached
// load: the value was written by the previous launch and only changes once this block's
// whole group has announced its leave.
__device__ __forceinline__ void need_tag(ParamsPtr p, Ctx &ctx)
{
    if (!ctx.have_tag) {
        ctx.tag = *(const volatile unsigned *)(p->epoch + (blockIdx.x % kGroups) * kCtlStride);
        ctx.have_tag = true;
    }
}

// Takes the block's next entry from its group's queue (calls longer than one round only).
// Items that never wait for other items ask when they start, so that the answer is there
// when they end.  Items that wait (conv items for the estimator, gen and gsum items for the
// pool sums) ask only after their wait: an entry reserved by a waiting block could be the
// very item it is waiting for.
__device__ __forceinline__ void claim_next(ParamsPtr p, Ctx &ctx)
{
    if (p->dynamic && opaque_tid() == kThreads - 1)
        ctx.claim = __hip_atomic_fetch_add(p->queue + (blockIdx.x % kGroups) * kCtlStride, 1u, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
}

// Called once the loads of the block's last item are in flight: announce the leave, so the
// atomic's round trip is over long before the block ends.
__device__ __forceinline__ void announce_leave(ParamsPtr p, Ctx &ctx)
{
    if (ctx.last_item && !ctx.announced) {
        need_tag(p, ctx);
        // Every wavefront's copy of the tag must have arrived before the announcement can be
        // seen: once the whole group has announced, the group's counter advances.
        asm volatile("" ::"v"(ctx.tag) : "memory");
        __syncthreads();
        if (threadIdx.x == kThreads - 1)
            ctx.left = __hip_atomic_fetch_add(p->done + (blockIdx.x % kGroups) * kCtlStride, 1u,
                                              __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ctx.announced = true;
    }
}

// The same, for a caller that has just passed a block barrier behind which every wavefront
// holds its copy of the call tag (need_tag called, and its load waited for, before it).
__device__ __forceinline__ void announce_leave_synced(unsigned *group_done, Ctx &ctx)
{
    if (ctx.last_item && !ctx.announced) {
        if (threadIdx.x == kThreads - 1)
            ctx.left = __hip_atomic_fetch_add(group_done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ctx.announced = true;
    }
}

// ---------------------------------------------------------------------------
// GAP partial sums (Eq. 4 line 2, first half).  A plane is cut into 64 x 32 pixel
// tiles.  Thread (tx, ty) = (t & 15, t >> 4) adds pixels (2*ty + a, 4*tx + q) of the
// tile for a, then q, ascending (pixels outside the image count as 0), then the
// wavefront tree adds the lanes and thread 0 the four wavefronts in order.  The order
// is the same whether the pixels come from global memory (pool item) or from a conv
// item's LDS tile, and depends on H and W only - so a batch reproduces its images run
// alone, and esc_dynkernel_gen reproduces the DK of the forward bit for bit.
// ---------------------------------------------------------------------------
template <int NB>
__device__ __forceinline__ void pool_finish(u64 *pool_box, const float (&s)[NB], const unsigned (&box)[NB],
                                            const bool (&have)[NB], uint32_t tag, float *s_red)
{
    // NB tiles at once (s_red holds 4 * NB floats): every tile's four wavefront totals, one
    // barrier, then thread b adds tile b's totals in ascending order and publishes the sum.
    // The caller keeps s_red untouched until the block's next barrier.
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const float w = wave_sum(s[b]);
        if ((threadIdx.x & 63) == 0) s_red[b * (kThreads / 64) + (threadIdx.x >> 6)] = w;
    }
    __syncthreads();
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        if ((int)threadIdx.x == b && have[b]) {
            float t = s_red[b * (kThreads / 64)];
#pragma unroll
            for (int w = 1; w < kThreads / 64; ++w) t += s_red[b * (kThreads / 64) + w];
            box_put(pool_box + box[b], t, tag);
        }
    }
}

// A pool item covers kPoolBatch consecutive pool tiles: all their loads go out together
// (no condition around a load - the compiler would wait for each guarded load before the
// next; addresses are clamped into the plane and what lies outside is zeroed afterwards),
// then each tile's sum is formed and published as if it were alone.
template <typename T>
__device__ __forceinline__ Ctx pool_item(ParamsPtr p, Ctx ctx, unsigned item)
{
    float *s_red = g_red;
    const int H = p->H, W = p->W;
    const int tid = opaque_tid();
    const int tx = tid & 15, ty = tid >> 4;
    const unsigned first = item * kPoolBatch, ntiles = p->n_pool_tiles;
    float v[kPoolBatch][2][4];
#pragma unroll
    for (int b = 0; b < kPoolBatch; ++b) {
        const bool have = first + b < ntiles;
        const unsigned tile = have ? first + b : ntiles - 1;
        const unsigned nc = fdiv(tile, p->div_ptiles.mul, p->div_ptiles.shift);
        const unsigned t = tile - nc * (unsigned)p->ptiles;
        const unsigned pty = fdiv(t, p->div_ptiles_x.mul, p->div_ptiles_x.shift), ptx = t - pty * (unsigned)p->ptiles_x;
        const unsigned n = fdiv(nc, p->div_ca.mul, p->div_ca.shift);
        const unsigned c = nc - n * (unsigned)p->Ca;
        const T *plane = (const T *)p->x + ((size_t)n * p->C + c) * (size_t)H * (size_t)W;
        const int gx = (int)ptx * kPoolTileW + 4 * tx, gy = (int)pty * kPoolTileH + 2 * ty;
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            if (p->conv_ld_vec) {  // W % 4 == 0 and an aligned base: the four pixels are in or out together
                const int ry = gy + a < H ? gy + a : H - 1, cx = gx < W ? gx : W - 4;
                load4(plane + (size_t)ry * W + cx, v[b][a]);
                const bool in = gy + a < H && gx < W;
#pragma unroll
                for (int q = 0; q < 4; ++q) v[b][a][q] = in ? v[b][a][q] : 0.f;
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    v[b][a][q] = 0.f;
                    if (gy + a < H && gx + q < W) v[b][a][q] = to_f32(plane[(size_t)(gy + a) * W + gx + q]);
                }
            }
        }
    }
    need_tag(p, ctx);
    announce_leave(p, ctx);
    float sums[kPoolBatch];
    unsigned box[kPoolBatch];
    bool have[kPoolBatch];
#pragma unroll
    for (int b = 0; b < kPoolBatch; ++b) {
        float s = 0.f;
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int q = 0; q < 4; ++q) s += v[b][a][q];
        sums[b] = s;
        box[b] = first + b;
        have[b] = first + b < ntiles;
    }
    pool_finish<kPoolBatch>(p->pool_box, sums, box, have, ctx.tag, s_red);
    return ctx;
}

// ---------------------------------------------------------------------------
// The kernel estimator (Eq. 4 line 2, second half) of image n.  The GAP of a
// channel is finished in one fixed order everywhere: lane l of a wavefront adds
// pool tiles l, l+64, ... ascending, then the wavefront tree adds the lanes.  Then
// the estimator, one output per thread.  A gen item publishes all 9*C_a outputs;
// when an image has few pool tiles the conv items skip that hop and derive their
// own nine values with the same arithmetic.
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

// The same for a weight row and an input vector that both sit in LDS.
typedef const __attribute__((address_space(3))) float *LdsFloats;
__device__ __forceinline__ float dot_row_lds(const float *w_, const float *in_, int K, float bias)
{
    LdsFloats w = (LdsFloats)w_, in = (LdsFloats)in_;
    float s = bias;
    for (int k0 = 0; k0 < K; k0 += 16) {  // operands first, so that their latencies overlap
        float wv[16], iv[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int k = k0 + u < K ? k0 + u : K - 1;
            wv[u] = w[k];
            iv[u] = in[k];
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) s = k0 + u < K ? fmaf(wv[u], iv[u], s) : s;
    }
    return s;
}

// The same with 16-byte LDS reads, for rows whose length is a multiple of four and that
// start on 16-byte boundaries (w_) - a quarter of the read instructions, and threads that
// read consecutive packed rows meet in far fewer banks.  Same products, same order.
__device__ __forceinline__ float dot_row_lds_vec(const float *w_, const float *in_, int K, float bias)
{
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    typedef const __attribute__((address_space(3))) f32x4 *LdsFloat4s;
    LdsFloat4s w = (LdsFloat4s)w_, in = (LdsFloat4s)in_;
    float s = bias;
    for (int k0 = 0; k0 < K; k0 += 16) {
        f32x4 wv[4], iv[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int q = k0 + 4 * v < K ? (k0 >> 2) + v : (K >> 2) - 1;
            wv[v] = w[q];
            iv[v] = in[q];
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const bool on = k0 + 4 * v < K;  // K % 4 == 0: a group of four is in or out as a whole
            s = on ? fmaf(wv[v].x, iv[v].x, s) : s;
            s = on ? fmaf(wv[v].y, iv[v].y, s) : s;
            s = on ? fmaf(wv[v].z, iv[v].z, s) : s;
            s = on ? fmaf(wv[v].w, iv[v].w, s) : s;
        }
    }
    return s;
}

// Channel means from the staged partial sums of a round that starts at channel c0.  The
// order of the additions depends on the tile count alone.  Many tiles: wavefront w takes
// channels w, w+4, ... < gc; lane l adds tiles l, l+64, ... ascending, then the wavefront
// tree.
__device__ __forceinline__ void sum_staged(const float *s_part, int ntile, int gc, int c0, float hw, float *s_g)
{
    if (ntile <= 64) {
        // few tiles: a row of 16 lanes per channel, sixteen channels of the block at once;
        // lane r adds tiles r, r+16, ... ascending, then the row's running sum
        LdsFloats part = (LdsFloats)s_part;
        const int tid = opaque_tid();
        const int r = tid & 15;
        for (int cg = tid >> 4; cg < gc; cg += kThreads / 16) {
            float s = 0.f;
            for (int k = r; k < ntile; k += 16) s += part[cg * ntile + k];
            s = row_sum(s);
            if (r == 15) s_g[c0 + cg] = s / hw;
        }
        return;
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int cg = wave; cg < gc; cg += kThreads / 64) {
        float s = 0.f;
        for (int k = lane; k < ntile; k += 64) s += s_part[cg * ntile + k];
        s = wave_sum(s);
        if (lane == 0) s_g[c0 + cg] = s / hw;
    }
}

// Whole block: waits for image n's pool mailboxes (staged through s_part), leaves the
// pooled means in s_g and (two-layer estimator) the hidden activations in s_t.  Ends
// with a barrier.
__device__ __forceinline__ void estimator_front(ParamsPtr p, uint32_t tag, unsigned n, int c_first, int c_end,
                                                bool with_hidden, float *s_part, float *s_g, float *s_t)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ntile = p->ptiles, Ca = p->Ca;
    const u64 *img_boxes = p->pool_box + (size_t)n * Ca * ntile;
    u64 polled[kStagePerThread];
    if (ntile <= kStage) {
        const int G = kStage / ntile;  // whole channels per round
        for (int c0 = c_first; c0 < c_end; c0 += G) {
            const int gc = c_end - c0 < G ? c_end - c0 : G;
            boxes_to_lds(img_boxes + (size_t)c0 * ntile, gc * ntile, s_part, tag, p->err, polled, false);
            __syncthreads();
            sum_staged(s_part, ntile, gc, c0, p->hw, s_g);
            __syncthreads();
        }
    } else {
        // a channel has more tiles than fit: kStage at a time; kStage % 64 == 0 keeps every
        // tile on the lane its index selects
        for (int c = c_first; c < c_end; ++c) {
            float s = 0.f;
            for (int k0 = 0; k0 < ntile; k0 += kStage) {
                const int cnt = ntile - k0 < kStage ? ntile - k0 : kStage;
                boxes_to_lds(img_boxes + (size_t)c * ntile + k0, cnt, s_part, tag, p->err, polled, false);
                __syncthreads();
                if (wave == 0)
                    for (int k = lane; k < cnt; k += 64) s += s_part[k];
                __syncthreads();
            }
            if (wave == 0) {
                s = wave_sum(s);
                if (lane == 0) s_g[c] = s / p->hw;
            }
        }
        __syncthreads();
    }
    if (with_hidden && p->hidden > 0) {
        for (int m = threadIdx.x; m < p->hidden; m += kThreads)
            s_t[m] = gelu_erf(dot_row(p->w_down + (size_t)m * Ca, s_g, Ca, p->b_down ? p->b_down[m] : 0.f));
        __syncthreads();
    }
}

// One thread: estimator output o (= DK entry c*9 + i*3 + j) from what estimator_front left.
__device__ __forceinline__ float estimator_out(ParamsPtr p, int o, const float *s_g, const float *s_t)
{
    const float *in = p->hidden > 0 ? s_t : s_g;
    const int K = p->hidden > 0 ? p->hidden : p->Ca;
    return dot_row(p->w_up + (size_t)o * K, in, K, p->b_up ? p->b_up[o] : 0.f);
}

__device__ __forceinline__ Ctx gen_item(ParamsPtr p, Ctx ctx, unsigned n)
{
    float *s_part = g_part, *s_g = g_g, *s_t = g_t;
    need_tag(p, ctx);
    announce_leave(p, ctx);
    // Small estimators (one output per thread, rows of at most 16 weights): the weights are
    // fetched now, while the pool sums are still being waited for, so that what follows the
    // wait is arithmetic only.  Same products in the same order as dot_row.
    constexpr int kRow = 16;
    const int Ca = p->Ca, hidden = p->hidden, K = hidden > 0 ? hidden : Ca;
    const bool pre = K <= kRow && Ca <= kRow && 9 * Ca <= kThreads && hidden <= kThreads;
    const int o1 = (int)threadIdx.x;
    float wu[kRow], wd[kRow], bu = 0.f, bd = 0.f;
    if (pre) {
#pragma unroll
        for (int k = 0; k < kRow; ++k) {
            wu[k] = (o1 < 9 * Ca && k < K) ? p->w_up[(size_t)o1 * K + k] : 0.f;
            wd[k] = (o1 < hidden && k < Ca) ? p->w_down[(size_t)o1 * Ca + k] : 0.f;
        }
        if (o1 < 9 * Ca && p->b_up) bu = p->b_up[o1];
        if (o1 < hidden && p->b_down) bd = p->b_down[o1];
    }
    estimator_front(p, ctx.tag, n, 0, Ca, !pre, s_part, s_g, s_t);
    if (pre) {
        if (hidden > 0) {
            if (o1 < hidden) {
                float s = bd;
#pragma unroll
                for (int k = 0; k < kRow; ++k)
                    if (k < Ca) s = fmaf(wd[k], s_g[k], s);
                s_t[o1] = gelu_erf(s);
            }
            __syncthreads();
        }
        if (o1 < 9 * Ca) {
            const float *in = hidden > 0 ? s_t : s_g;
            float s = bu;
#pragma unroll
            for (int k = 0; k < kRow; ++k)
                if (k < K) s = fmaf(wu[k], in[k], s);
            const size_t idx = (size_t)n * 9 * Ca + o1;
            box_put(p->dk_box + idx, s, ctx.tag);
            if (p->dk_out) p->dk_out[idx] = s;
        }
    } else {
        for (int o = threadIdx.x; o < 9 * Ca; o += kThreads) {
            const float s = estimator_out(p, o, s_g, s_t);
            const size_t idx = (size_t)n * 9 * Ca + o;
            box_put(p->dk_box + idx, s, ctx.tag);
            if (p->dk_out) p->dk_out[idx] = s;
        }
    }
    claim_next(p, ctx);
    return ctx;
}

// ---------------------------------------------------------------------------
// The estimator items of the kernel flavour for channel-mean calls and for estimators
// beyond the small ones (forward_kernel<..., true>).  Kept apart from the items above so
// that the code of the other flavour - the one the short calls use - stays what it is.
// ---------------------------------------------------------------------------

// gsum item: the mean of one (image, channel) plane from its pool mailboxes, with the
// additions in the order every other path uses, published in the channel's mean mailbox.
__device__ __forceinline__ Ctx gsum_item(ParamsPtr p, Ctx ctx, unsigned nc)
{
    float *s_part = g_part, *s_g = g_g, *s_t = g_t;
    need_tag(p, ctx);
    announce_leave(p, ctx);
    const unsigned n = fdiv(nc, p->div_ca.mul, p->div_ca.shift);
    const int c = (int)(nc - n * (unsigned)p->Ca);
    estimator_front(p, ctx.tag, n, c, c + 1, false, s_part, s_g, s_t);
    if (threadIdx.x == 0) box_put(p->g_box + nc, s_g[c], ctx.tag);
    claim_next(p, ctx);
    return ctx;
}

// gen item of image n: the means come from the pool mailboxes (as in gen_item) or, in a
// channel-mean call, from the gsum items' mailboxes.  All threads together stage the
// estimator's weights in the tile's LDS (no conv item is running in this block): the first
// layer's before the wait, afterwards the output rows, as many at a time as fit.  Read row
// after row from memory by the few threads that use them, these weights cost the block ten
// microseconds and more (measured with C_a = 48 and a hidden layer of 24).  Same products
// in the same order as dot_row, so DK has the same bits whichever item computes it.
__device__ __forceinline__ Ctx gen_item_staged(ParamsPtr p, Ctx ctx, unsigned n, bool from_means)
{
    float *s_part = g_part, *s_g = g_g, *s_t = g_t, *s_w = g_tile;
    need_tag(p, ctx);
    announce_leave(p, ctx);
    const int Ca = p->Ca, hidden = p->hidden, K = hidden > 0 ? hidden : Ca;
    const int o1 = (int)threadIdx.x;
    // the staging area holds the whole first layer and, behind it, at least 64 output rows
    const int n_dn = hidden * Ca;
    const bool staged = n_dn + 64 * K <= kLdsTileFloats;
    constexpr int kFlight = 24;  // loads a thread has in flight
    auto stage = [&](const float *src, int count, float *dst) {
        for (int i0 = 0; i0 < count; i0 += kFlight * kThreads) {
            float t[kFlight];
#pragma unroll
            for (int u = 0; u < kFlight; ++u) {
                const int i = i0 + u * kThreads + o1;
                t[u] = src[i < count ? i : count - 1];
            }
#pragma unroll
            for (int u = 0; u < kFlight; ++u) {
                const int i = i0 + u * kThreads + o1;
                if (i < count) dst[i] = t[u];
            }
        }
    };
    float *s_rows = s_w + n_dn;
    const bool vec_rows = (K & 3) == 0 && (n_dn & 3) == 0;  // rows of s_rows are 16-byte aligned
    const int rows = !staged ? 0 : (kLdsTileFloats - n_dn) / K < kThreads ? (kLdsTileFloats - n_dn) / K : kThreads;
    float bd = 0.f;
    if (staged) {  // first layer and the first round of output rows, before the wait
        if (hidden > 0) {
            if (p->b_down) bd = p->b_down[o1 < hidden ? o1 : 0];
            stage(p->w_down, n_dn, s_w);
        }
        stage(p->w_up, (9 * Ca < rows ? 9 * Ca : rows) * K, s_rows);
    }
    if (from_means) {
        // the gsum items have finished the channels' means: collect them (C_a <= kStage)
        u64 polled[kStagePerThread];
        boxes_to_lds(p->g_box + (size_t)n * Ca, Ca, s_part, ctx.tag, p->err, polled, false);
        __syncthreads();
        for (int k = o1; k < Ca; k += kThreads) s_g[k] = s_part[k];
        __syncthreads();
    } else {
        estimator_front(p, ctx.tag, n, 0, Ca, false, s_part, s_g, s_t);
    }
    if (hidden > 0) {
        for (int m = o1; m < hidden; m += kThreads)
            s_t[m] = gelu_erf(staged ? dot_row_lds(s_w + m * Ca, s_g, Ca, bd)
                                     : dot_row(p->w_down + (size_t)m * Ca, s_g, Ca, p->b_down ? p->b_down[m] : 0.f));
        __syncthreads();
    }
    if (staged) {
        const float *in = hidden > 0 ? s_t : s_g;
        for (int r0 = 0; r0 < 9 * Ca; r0 += rows) {  // block-uniform
            const int nr = 9 * Ca - r0 < rows ? 9 * Ca - r0 : rows;
            if (r0 > 0) {
                stage(p->w_up + (size_t)r0 * K, nr * K, s_rows);
                __syncthreads();
            }
            if (o1 < nr) {
                const float bias = p->b_up ? p->b_up[r0 + o1] : 0.f;
                const float sacc = vec_rows ? dot_row_lds_vec(s_rows + o1 * K, in, K, bias)
                                            : dot_row_lds(s_rows + o1 * K, in, K, bias);
                const size_t idx = (size_t)n * 9 * Ca + r0 + o1;
                box_put(p->dk_box + idx, sacc, ctx.tag);
                if (p->dk_out) p->dk_out[idx] = sacc;
            }
            __syncthreads();  // the rows' area is reused
        }
    } else {
        for (int o = o1; o < 9 * Ca; o += kThreads) {
            const float sacc = estimator_out(p, o, s_g, s_t);
            const size_t idx = (size_t)n * 9 * Ca + o;
            box_put(p->dk_box + idx, sacc, ctx.tag);
            if (p->dk_out) p->dk_out[idx] = sacc;
        }
    }
    claim_next(p, ctx);
    return ctx;
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
    static constexpr int ROWS = RY + KS - 1;      // tile rows a thread walks through
    static constexpr bool UNROLL = KS <= 17;
};

// bf16 storage with Ks <= 17: the tap loop runs on the matrix cores.  One row of the
// depth-wise kernel applied to 16 neighbouring outputs of an image row is a product with a
// banded (Toeplitz) matrix: out[x0 + m] += sum_k T_i[m][k] * x[row + i][t0 + k], with
// T_i[m][k] = LK[i][k - m - S0] inside the band and 0 outside, and 16 + Ks - 1 <= 32 input
// columns are exactly the K of one v_mfma_f32_16x16x32_bf16.  A = T_i (16 output columns x
// 32 tile columns), B = 32 tile columns x 16 image rows, so the instruction yields a 16 x 16
// block of outputs for kernel row i; Ks of them, the tile rows moving down by one each time,
// finish the block.  (60 % of the products are with zeros of the band; the matrix cores
// are 17 times faster than the two-tap dot instruction this loop used to run on, whose
// rate bounded these calls.)
//
// LDS layout: the tile is cut into pieces of 8 columns (16 bytes) and stored piece column
// after piece column - element (r, t) at ((t / 8) * HRP + r) * 8 + t % 8 - so that the 16
// lanes that read one B operand's rows at one piece column read 256 consecutive bytes (the
// LDS delivers 16-byte reads at full rate only then; row-major with any pitch runs at half).
// HRP is odd: pieces of neighbouring columns start on different banks.  Tile column t is
// image column x0 - PH - A + t (A pads the halo to 8 columns, so that a piece is 16 aligned
// bytes of memory where the image's width and base allow 16-byte fetches); all 80
// columns of every row are written for every item, because what lies beyond the halo is
// multiplied by the zeros of the band and must not be stale.  Lane (m, kg) = (l % 16, l / 16)
// of an A operand holds T_i[m][8 kg ... 8 kg + 7], which depends on 8 kg - m alone: the 40
// distinct operands per kernel row are staged behind the tile, 16 bytes each.
template <int KS, int RY>
struct MatrixGeom {
    using G = ConvGeom<KS, RY>;
    static constexpr int A = (8 - G::PH % 8) % 8;  // the halo starts a multiple of 8 columns left of the tile's outputs
    static constexpr int S0 = A + G::OFF;        // tile column of tap 0 for output column 0
    static constexpr int COLS = kTileW + 16;     // 80 tile columns
    static constexpr int NCH = COLS / 4;         // 4-element chunks per tile row
    static constexpr int HRP = G::HR | 1;        // rows per piece column (odd)
    static constexpr int TILE_WORDS = (COLS / 8) * HRP * 4;
    static constexpr int ND = 40;                // 8 kg - m + 15 = 0 ... 39
    static constexpr int TBL_WORDS = KS * ND * 4;
    // After the tap loop the table's place takes the output tile on its way to memory: bf16,
    // row-major, OP words per row (the results leave the matrix cores as 16 rows x 4 columns
    // per lane group, which would be stored in 32-byte runs; passed through LDS, sixteen
    // lanes store a whole 128-byte row segment).  The odd multiple of two words keeps the
    // sixteen rows a wavefront writes at once on different banks.
    static constexpr int OP = kTileW / 2 + 2;
    static constexpr int OUT_WORDS = G::TH * OP;
    static_assert(KS > 17 || G::HC + A <= COLS, "the halo does not fit in 80 tile columns");
    static_assert(KS > 17 || 15 + (KS - 1) + S0 <= 31, "a block of 16 outputs needs more than 32 tile columns");
    static_assert(KS > 17 || TILE_WORDS + (TBL_WORDS > OUT_WORDS ? TBL_WORDS : OUT_WORDS) <= kLdsTileFloats,
                  "LDS pool too small");  // (larger kernels do not take this path)
    // word (two bf16) `wi` of tile row r
    __device__ static __forceinline__ int word(int r, int wi) { return ((wi >> 2) * HRP + r) * 4 + (wi & 3); }
};

// where a conv item lies
struct ConvWhere {
    unsigned n, nc;
    int c, txi, tyi, x0, y0;
    size_t plane_off;
};
template <int TH>
__device__ __forceinline__ ConvWhere conv_where(ParamsPtr p, unsigned item)
{
    ConvWhere w;
    const unsigned b1 = fdiv(item, p->div_tiles_x.mul, p->div_tiles_x.shift);
    w.txi = (int)(item - b1 * p->div_tiles_x.d);
    w.nc = fdiv(b1, p->div_tiles_y.mul, p->div_tiles_y.shift);
    w.tyi = (int)(b1 - w.nc * p->div_tiles_y.d);
    w.n = fdiv(w.nc, p->div_ca.mul, p->div_ca.shift);
    w.c = (int)(w.nc - w.n * (unsigned)p->Ca);
    w.plane_off = ((size_t)w.n * p->C + w.c) * (size_t)p->H * (size_t)p->W;
    w.x0 = w.txi * kTileW;
    w.y0 = w.tyi * TH;
    return w;
}

template <int KS, int RY, typename T, bool ADD>
__device__ __forceinline__ Ctx conv_item(ParamsPtr p, Ctx ctx, unsigned item_in)
{
    using G = ConvGeom<KS, RY>;
    static_assert(G::TILE_FLOATS <= kLdsTileFloats && G::W_FLOATS <= kLdsWeightFloats, "LDS pool too small");
    float *tile = g_tile, *wl = g_wl, *s_dk = g_small, *s_part = g_part, *s_g = g_g, *s_t = g_t;
    constexpr int PH = G::PH, OFF = G::OFF, TH = G::TH, HR = G::HR, HC = G::HC, PITCH = G::PITCH,
                  NV = G::NV, WP = G::WP;
    // bf16 storage and Ks <= 17: bf16 tile in pieces of 8 columns, tap loop on the matrix cores (MatrixGeom)
    constexpr bool kMatrix = std::is_same<T, bf16_t>::value && G::UNROLL;
    using MG = MatrixGeom<KS, RY>;
    uint32_t *tile_d = reinterpret_cast<uint32_t *>(g_tile), *tbl_d = tile_d + MG::TILE_WORDS;
    uint16_t *tile_h = reinterpret_cast<uint16_t *>(g_tile);
    const int H = p->H, W = p->W;

    // ---- phase 1: fetch the halo tile and the channel's weights into LDS ----
    const unsigned item = opaque_u(item_in);
    const ConvWhere wa = conv_where<TH>(p, item);
    const unsigned n = wa.n, nc = wa.nc;
    const int c = wa.c, txi = wa.txi, tyi = wa.tyi, x0 = wa.x0, y0 = wa.y0;
    const T *xp = (const T *)p->x + wa.plane_off;

    // this channel's weights, asked for right behind the tile's loads (results return in order:
    // in front of them, the tile would wait for the weights as well)
    constexpr int KW = (KS * KS + kThreads - 1) / kThreads;
    const float *lkc = p->lk + (size_t)c * p->lk_cstride;
    // (thread indices are taken afresh in every phase, so that nothing derived from them
    // is computed once per kernel and then held in registers through all items)
    const int tid1 = opaque_tid();
    float wreg[KW];
    auto load_weights = [&]() {
#pragma unroll
        for (int m = 0; m < KW; ++m) {
            const int idx = m * kThreads + tid1;
            wreg[m] = idx < KS * KS ? lkc[idx] : 0.f;
        }
    };

    // Carried copy (Eq. 4 lines 1 and 4): this item's share of the image's pass-through range
    // - up to kCarryGrains grains of 16 bytes per thread - is asked for once the tile has
    // landed and its pool sums are out, travels while the tile is multiplied, and is stored
    // after the tap loop, where the item would otherwise only wait for the estimator.  The
    // copy thus has no block of its own.  Earlier blocks' shares asked for ahead of the tile
    // delay the tiles of later blocks, and with them the pool sums every estimator waits for;
    // asked for after the band table they come back too late for the store.  (Measured at
    // 360 x 640 and 64 x 64 x 64 against: right behind the tile loads, behind the fill
    // barrier, after the band table, after the loop, before the tile in every other block.)
    // Buffer accesses: the resources end with the share, so grains beyond it read as nothing
    // and their stores are dropped, without a branch.
    constexpr bool kCarry = conv_carries(KS, RY, std::is_same<T, bf16_t>::value);
    constexpr int kCarryN = kCarry ? kCarryGrains : 1;
    CarryRsrc carry_dst = __builtin_amdgcn_make_buffer_rsrc(nullptr, 0, 0, kRawBufferFlags);
    u32x4 carry_v[kCarryN] = {};
    auto carry_load = [&]() {
        if constexpr (kCarry) {
            const unsigned per_plane = p->div_tiles_x.d * p->div_tiles_y.d;
            const size_t j = (size_t)c * per_plane + (size_t)tyi * p->div_tiles_x.d + (size_t)txi;
            const size_t share = (size_t)p->carry_g * kGrain;
            const size_t begin = j * share;
            const size_t lim = p->copy_off;  // what the conv items carry ends here
            const size_t len = begin < lim ? (lim - begin < share ? lim - begin : share) : 0;
            const size_t base = (size_t)n * p->img_bytes + p->idt_off + begin;
            const CarryRsrc src =
                __builtin_amdgcn_make_buffer_rsrc((void *)((const char *)p->x + base), 0, (int)len, kRawBufferFlags);
            carry_dst = __builtin_amdgcn_make_buffer_rsrc((void *)((char *)p->out + base), 0, (int)len, kRawBufferFlags);
            const int voff = opaque_tid() * 16;
#pragma unroll
            for (int r = 0; r < kCarryN; ++r)
                carry_v[r] = __builtin_amdgcn_raw_buffer_load_b128(src, voff + r * (int)kGrain, 0, kBufferNt);
        }
    };
    auto carry_store = [&]() {
        if constexpr (kCarry) {
            const int voff = opaque_tid() * 16;
#pragma unroll
            for (int r = 0; r < kCarryN; ++r)
                __builtin_amdgcn_raw_buffer_store_b128(carry_v[r], carry_dst, voff + r * (int)kGrain, 0, kBufferNt);
        }
    };

    // halo tile -> LDS, zero outside the image
    if (kMatrix && p->conv_ld_vec == 2) {
        // bf16, W % 8 == 0 and a 16-byte aligned base: whole pieces of 8 columns (each lies
        // entirely inside or outside the image), all loads in flight before the first LDS write
        if constexpr (kMatrix) {
            constexpr int NP8 = MG::COLS / 8;
            constexpr int TOT = HR * NP8;
            constexpr int K = (TOT + kThreads - 1) / kThreads;
            const int g0 = x0 - PH - MG::A;
            u32x4 raw[K];
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const int q = k * kThreads + tid1;
                const int r = q / NP8, j = q - r * NP8;
                const int gy = y0 - PH + r, gx = g0 + 8 * j;
                const bool in = q < TOT && gy >= 0 && gy < H && gx >= 0 && gx < W;
                raw[k] = u32x4{0u, 0u, 0u, 0u};
                if (in) raw[k] = *reinterpret_cast<const u32x4 *>(xp + (size_t)gy * W + gx);
            }
            load_weights();
        if (p->pool_mode != kPoolNone || ctx.last_item) need_tag(p, ctx);
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const int q = k * kThreads + tid1;
                const int r = q / NP8, j = q - r * NP8;
                if (q < TOT) *reinterpret_cast<u32x4 *>(tile_d + MG::word(r, 4 * j)) = raw[k];
            }
        }
    } else if (p->conv_ld_vec) {
        // W % 4 == 0 and an aligned base: fetch whole 4-element chunks aligned in global
        // memory (each lies entirely inside or outside the image), all loads in flight
        // before the first LDS write.  A chunk lands at LDS column 4j - A.
        constexpr int A = kMatrix ? MG::A : (4 - PH % 4) % 4;
        constexpr int NCH = kMatrix ? MG::NCH : (HC + A + 3) / 4;
        constexpr int TOT = HR * NCH;
        constexpr int K = (TOT + kThreads - 1) / kThreads;
        const int g0 = x0 - PH - A;
        float v[K][4];
        uint2 raw[K];
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const int q = k * kThreads + tid1;
            const int r = q / NCH, j = q - r * NCH;
            const int gy = y0 - PH + r, gx = g0 + 4 * j;
            const bool in = q < TOT && gy >= 0 && gy < H && gx >= 0 && gx < W;
            if constexpr (kMatrix) {
                raw[k] = make_uint2(0u, 0u);
                if constexpr (std::is_same<T, bf16_t>::value)
                    if (in) raw[k] = load4_raw(xp + (size_t)gy * W + gx);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[k][e] = 0.f;
                if (in) load4(xp + (size_t)gy * W + gx, v[k]);
            }
        }
        load_weights();
        if (p->pool_mode != kPoolNone || ctx.last_item) need_tag(p, ctx);
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const int q = k * kThreads + tid1;
            const int r = q / NCH, j = q - r * NCH;
            if constexpr (kMatrix) {  // the chunk is words 2j, 2j + 1 of row r
                if (q < TOT) *reinterpret_cast<uint2 *>(tile_d + MG::word(r, 2 * j)) = raw[k];
            } else if (q < TOT) {
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
    } else if constexpr (kMatrix) {
        // element by element, all 80 columns of every row (what lies beyond the halo is
        // multiplied by the zeros of the band and must not be stale LDS)
        if constexpr (std::is_same<T, bf16_t>::value) {
            for (int idx = tid1; idx < HR * MG::COLS; idx += kThreads) {
                const int r = idx / MG::COLS, cc = idx - r * MG::COLS;
                const int gy = y0 - PH + r, gx = x0 - PH - MG::A + cc;
                uint16_t v = 0;
                if (gy >= 0 && gy < H && gx >= 0 && gx < W) v = xp[(size_t)gy * W + gx].bits;
                tile_h[2 * MG::word(r, cc >> 1) + (cc & 1)] = v;
            }
        }
        load_weights();
        if (p->pool_mode != kPoolNone || ctx.last_item) need_tag(p, ctx);
    } else {
        for (int idx = tid1; idx < HR * HC; idx += kThreads) {
            const int r = idx / HC, cc = idx - r * HC;
            const int gy = y0 - PH + r, gx = x0 - PH + cc;
            float v = 0.f;
            if (gy >= 0 && gy < H && gx >= 0 && gx < W) v = to_f32(xp[(size_t)gy * W + gx]);
            tile[r * PITCH + cc] = v;
        }
        load_weights();
        if (p->pool_mode != kPoolNone || ctx.last_item) need_tag(p, ctx);
    }
#pragma unroll
    for (int m = 0; m < KW; ++m) {
        const int idx = m * kThreads + tid1;
        // (matrix path: the Ks x Ks weights as they lie in memory; the band table is made from them further down)
        if (idx < KS * KS) wl[kMatrix ? idx : (idx / KS) * WP + idx % KS] = wreg[m];
    }
    // (the call tag, asked for behind the tile, has arrived in this wavefront too)
    asm volatile("" ::"v"(ctx.tag));
    __syncthreads();
    // The leave is announced here: every wavefront of the block has its tile and its copy of
    // the call tag (the barrier above), and the announcing wavefront's atomic is then in
    // flight during the tap loop, which waits for no memory access.  Anywhere earlier, the
    // next wait for a load would wait for the atomic as well - results return in order; any
    // later, behind the pool mailbox's store, a wait for the tag would wait for that store's
    // round trip too.
    announce_leave_synced(p->done + (blockIdx.x % kGroups) * kCtlStride, ctx);

    const int tid2 = opaque_tid();
    const int tx = tid2 & 15, ty = tid2 >> 4;

    // Every conv item is resident (the host checked): publish the GAP partial sums of the
    // pool tiles this tile covers, straight from LDS, instead of reading the plane twice.
    if (p->pool_mode == kPoolFused) {
        constexpr int NPT = TH / kPoolTileH;  // pool tiles stacked in this conv tile
        static_assert(NPT <= kPoolBatch, "g_red holds kPoolBatch tiles");
        float sums[NPT];
        unsigned box[NPT];
        bool have[NPT];
#pragma unroll
        for (int h = 0; h < NPT; ++h) {
            const unsigned pty = (unsigned)tyi * NPT + h;
            float s = 0.f;
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                if constexpr (kMatrix) {  // the same four pixels, in the same order
                    const uint2 w2 = *reinterpret_cast<const uint2 *>(
                        tile_d + MG::word(h * kPoolTileH + 2 * ty + a + PH, 2 * tx + (PH + MG::A) / 2));
                    s += bf16_lo(w2.x);
                    s += bf16_hi(w2.x);
                    s += bf16_lo(w2.y);
                    s += bf16_hi(w2.y);
                } else {
                    const float *src = tile + (h * kPoolTileH + 2 * ty + a + PH) * PITCH + 4 * tx + PH;
#pragma unroll
                    for (int q = 0; q < 4; ++q) s += src[q];
                }
            }
            sums[h] = s;
            box[h] = (nc * (unsigned)p->ptiles) + pty * (unsigned)p->ptiles_x + (unsigned)txi;
            have[h] = (int)pty * kPoolTileH < H;  // block-uniform
        }
        pool_finish<NPT>(p->pool_box, sums, box, have, ctx.tag, g_red);
    }
    carry_load();
    if constexpr (kMatrix) {
        // The band table (MatrixGeom), made from the weights in LDS once the pool sums are
        // out (they are what the other blocks wait for): word idx holds the band's entries for
        // two neighbouring tile columns - kernel row i = idx / 160, operand d = (idx % 160) / 4,
        // columns k = 2 (idx % 4), + 1 of the operand's eight, i.e. taps j = d - 15 + k - S0.
        constexpr int KWP = (MG::TBL_WORDS + kThreads - 1) / kThreads;
#pragma unroll
        for (int m = 0; m < KWP; ++m) {
            const int idx = m * kThreads + tid2;
            int i = idx / (MG::ND * 4);
            const int rem = idx - i * (MG::ND * 4);
            const int ja = (rem >> 2) - 15 + 2 * (rem & 3) - MG::S0, jb = ja + 1;
            i = i < KS ? i : KS - 1;
            const float va = wl[i * KS + (ja < 0 ? 0 : ja >= KS ? KS - 1 : ja)];
            const float vb = wl[i * KS + (jb < 0 ? 0 : jb >= KS ? KS - 1 : jb)];
            const uint32_t ha = (ja >= 0 && ja < KS) ? f32_to_bf16_bits(va) : 0u;
            const uint32_t hb = (jb >= 0 && jb < KS) ? f32_to_bf16_bits(vb) : 0u;
            if (idx < MG::TBL_WORDS) tbl_d[idx] = ha | (hb << 16);
        }
        __syncthreads();
    }

    // What the DK phase will need is asked for ahead of it: the estimator weights this
    // channel needs (conv items that run the estimator themselves) before the tap loop, the
    // mailboxes (pool sums, channel means or DK itself) from inside it; the answers are
    // looked at after the loop, so that their round trips cost nothing.
    constexpr int kPer = (kDirectMaxBoxes + kPollThreads - 1) / kPollThreads;
    const bool from_boxes = p->dk_mode == kDkBoxes;  // a gen item publishes DK itself
    const bool means = p->dk_mode == kDkMeans;
    const bool direct = p->dk_mode == kDkDirect || means;  // this item runs the estimator
    const int nbox = from_boxes ? 9 : means ? p->Ca : p->Ca * p->ptiles;
    const u64 *img_boxes = from_boxes ? p->dk_box + (size_t)nc * 9
                           : means    ? p->g_box + (size_t)n * nbox
                                      : p->pool_box + (size_t)n * nbox;
    const int Kin = p->hidden > 0 ? p->hidden : p->Ca;
    const bool pre_w = direct && 9 * Kin <= kThreads && p->hidden * p->Ca <= kThreads;
    u64 early[kPer];
    float wup_r = 0.f, wdn_r = 0.f, bup_r = 0.f, bdn_r = 0.f;
    auto ask_early = [&]() {
        if (direct) {
#pragma unroll
            for (int u = 0; u < kPer; ++u) {
                const int f = tid2 + u * kPollThreads;
                early[u] = 0;
                if (!G::UNROLL && tid2 < kPollThreads && f < nbox)
                    early[u] = __hip_atomic_load(img_boxes + f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (pre_w) {
                if (tid2 < 9 * Kin) wup_r = p->w_up[(size_t)c * 9 * Kin + tid2];
                if (tid2 < p->hidden * p->Ca) wdn_r = p->w_down[tid2];
                if (tid2 < 9 && p->b_up) bup_r = p->b_up[c * 9 + tid2];
                if (tid2 < p->hidden && p->b_down) bdn_r = p->b_down[tid2];
            }
        }
    };

    // Asked again in one of the last steps of the tap loop (any earlier, and in a call of one
    // round the other blocks have not published yet): the answers travel while the loop ends.  The mailboxes' base is block-uniform and
    // waits in scalar registers; the per-thread addresses are made on the spot.
    const u64 *boxes_s = img_boxes;
    asm volatile("" : "+s"(boxes_s));
    auto ask_again = [&]() {
        // no branch here (one would split the loop body and cost registers): every thread
        // reads some mailbox of the image, whichever mode the call is in
        const int t = opaque_tid();
        const u64 *bx = boxes_s;
        // (threads beyond the image's mailboxes read their block group's counter line instead:
        // aimed at the last mailbox, a thousand blocks' idle lanes would queue on a few lines)
        const u64 *idle = reinterpret_cast<const u64 *>(p->epoch + (blockIdx.x % kGroups) * kCtlStride);
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const int f = t + u * kPollThreads;
            early[u] = __hip_atomic_load(f < nbox ? bx + f : idle, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    };

    float acc[RY][4];
#pragma unroll
    for (int oy = 0; oy < RY; ++oy)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[oy][q] = 0.f;

    const float *trow = tile + (ty * RY) * PITCH + 4 * tx;

    // The tap loop, software-pipelined by hand so that the register use is ours to decide:
    // while row r is multiplied, tile row r+1 is already on its way from LDS (two buffers),
    // and kernel row r - the only new one - arrives while the older kernel rows, held in
    // registers from the steps before, are applied first.  A scheduling barrier ends every
    // step so the compiler cannot pull later rows' loads up and run out of registers.
    // (The matrix path has a loop of its own, further down.)
    using XT = float;
    constexpr int NX = NV;    // values of a tile row per thread
    constexpr int NWT = KS;   // values of a kernel row
    auto load_x = [&](int r, XT *v) {
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
    };
    auto load_w = [&](int i, XT *w) {
        {
            const float *wsrc = wl + i * WP;
#pragma unroll
            for (int k = 0; k + 4 <= KS; k += 4) {
                const float4 f = *reinterpret_cast<const float4 *>(wsrc + k);
                w[k + 0] = f.x;
                w[k + 1] = f.y;
                w[k + 2] = f.z;
                w[k + 3] = f.w;
            }
#pragma unroll
            for (int k = KS & ~3; k < KS; ++k) w[k] = wsrc[k];
        }
    };
    auto fma_row = [&](float *a, const XT *w, const XT *v) {
#pragma unroll
        for (int j = 0; j < KS; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) a[q] = fmaf(w[j], v[j + q], a[q]);
    };
    // what may move across a step boundary: arithmetic only, not LDS traffic
    constexpr int kSchedNoLds = 0x1 | 0x2 | 0x4;

    // room for a second tile-row buffer?
    constexpr bool kTwoX = 2 * NX + RY * NWT + 4 * RY <= 96;
    XT X[kTwoX ? 2 : 1][NX];
    XT Wt[RY][NWT];  // kernel row i lives in slot i % RY while it is in use
    if (kTwoX) load_x(0, X[0]);
    auto step = [&](int r, int u) {  // u == r % RY, and RY is even
        XT *xc = X[kTwoX ? (u & 1) : 0];
        if (kTwoX) {
            if (r + 1 < G::ROWS) load_x(r + 1, X[(u + 1) & 1]);
        } else {
            load_x(r, xc);
        }
        if (r < KS) load_w(r, Wt[u]);
        if (r >= RY - 1 && r < KS) {
            // every output row of the thread takes part: interleave them tap by tap, oldest
            // kernel row first, so that 4*RY independent accumulators are in flight
#pragma unroll
            for (int j = 0; j < KS; ++j)
#pragma unroll
                for (int k = RY - 1; k >= 0; --k)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        acc[k][q] = fmaf(Wt[(u - k + RY) % RY][j], xc[j + q], acc[k][q]);
        } else {
#pragma unroll
            for (int k = RY - 1; k >= 0; --k) {  // output row k of this thread: kernel row r - k
                const int i = r - k;
                if (i >= 0 && i < KS) fma_row(acc[k], Wt[(u - k + RY) % RY], xc);
            }
        }
        __builtin_amdgcn_sched_barrier(kSchedNoLds);
    };
    // The tap loop is the one long stretch of pure arithmetic: it runs at the lowest
    // wavefront priority, everything else (issuing loads, the serial estimator code, the
    // stores) above it, so that the short latency-bound phases of one block are not starved
    // by the tap loops of the other blocks on the compute unit.
    __builtin_amdgcn_s_setprio(0);
    // The early requests go out before the loop (in its middle they cost the compiler so
    // many registers that it spills); whatever has not arrived by the end is asked for again.
    ask_early();
    if constexpr (kMatrix) {
        // The matrix path (MatrixGeom).  The tile's 4 * RY blocks of 16 x 16 outputs are dealt
        // to the four wavefronts, RY neighbouring blocks of one row of blocks each: block
        // b = wv * RY + t covers output rows 16 (b / 4) ... and columns 16 (b % 4) ...  Per
        // kernel row: one A operand (the band, shared by the wavefront's blocks) and one B
        // operand per block (lane (n, kg): tile row 16 (b / 4) + i + n, columns 16 (b % 4) +
        // 8 kg ... + 7), the next kernel row's operands in flight while this one's multiply.
        // The result: lane (n, g) of block t holds output row n, columns 4 g ... 4 g + 3.
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
        const int lane = tid2 & 63, b0 = (tid2 >> 6) * RY;
        const int nrow = lane & 15, kg = lane >> 4;
        const uint32_t *a_src = tbl_d + (8 * kg - nrow + 15) * 4;
        const uint32_t *b_src = tile_d + ((2 * (b0 & 3) + kg) * MG::HRP + 16 * (b0 >> 2) + OFF + nrow) * 4;
        auto load_a = [&](int i) { return *reinterpret_cast<const u32x4 *>(a_src + i * (MG::ND * 4)); };
        auto load_b = [&](int i, int t) { return *reinterpret_cast<const u32x4 *>(b_src + (2 * t * MG::HRP + i) * 4); };
        f32x4 macc[RY];
        u32x4 av[2], bv[2][RY];
        av[0] = load_a(0);
#pragma unroll
        for (int t = 0; t < RY; ++t) {
            macc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
            bv[0][t] = load_b(0, t);
        }
#pragma unroll
        for (int i = 0; i < KS; ++i) {
            if (i == (KS * 15) / 16) ask_again();
            if (i + 1 < KS) {
                av[(i + 1) & 1] = load_a(i + 1);
#pragma unroll
                for (int t = 0; t < RY; ++t) bv[(i + 1) & 1][t] = load_b(i + 1, t);
            }
#pragma unroll
            for (int t = 0; t < RY; ++t)
                macc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av[i & 1]),
                                                                  __builtin_bit_cast(bf16x8, bv[i & 1][t]), macc[t], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(kSchedNoLds);
        }
        carry_store();
#pragma unroll
        for (int t = 0; t < RY; ++t)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[t][q] = macc[t][q];
    } else if (G::UNROLL) {
#pragma unroll
        for (int r0 = 0; r0 < G::ROWS; r0 += RY)
#pragma unroll
            for (int u = 0; u < RY; ++u)
                if (r0 + u < G::ROWS) {
                    if (r0 + u == (G::ROWS * 15) / 16) ask_again();
                    step(r0 + u, u);
                }
    } else {
        // Large kernels: a loop, two rows per trip; the kernel rows are re-read from LDS for
        // every output row instead of being held (they would not fit in the registers).
#pragma unroll 2
        for (int r = 0; r < G::ROWS; ++r) {
            XT xr[NX];
            load_x(r, xr);
#pragma unroll
            for (int k = 0; k < RY; ++k) {
                const int i = r - k;
                if (i >= 0 && i < KS) {
                    XT wr[NWT];
                    load_w(i, wr);
                    fma_row(acc[k], wr, xr);
                }
            }
            __builtin_amdgcn_sched_barrier(0);  // one row's loads at a time: the registers are few
        }
    }
    __builtin_amdgcn_s_setprio(kPrioHigh);

    // ---- phase 3: DK and the stores, located afresh (see opaque_u) ----
    const ConvWhere wd = conv_where<TH>(p, opaque_u(item_in));
    const int tid_d = opaque_tid();
    const int tx_d = tid_d & 15, ty_d = tid_d >> 4;
    const float *trow_d = tile + (ty_d * RY) * PITCH + 4 * tx_d;
    // matrix path: the wavefront's first block, the lane's output row inside a block and its group of four columns
    const int mb0 = (tid_d >> 6) * RY, mrow = tid_d & 15, mg4 = (tid_d & 63) >> 4;
    T *op = (T *)p->out + ((size_t)wd.n * p->out_c + wd.c) * (size_t)p->H * (size_t)p->W;  // out may have fewer channels than x

    if (p->dk_mode != kDkNone) {
        const size_t dk_idx = ((size_t)wd.n * p->Ca + wd.c) * 9;
        float *s_wup = s_part + kDirectMaxBoxes, *s_wdn = s_part + kDirectMaxBoxes + kThreads;
        if (direct) {
            // same arithmetic, in the same order, as estimator_front + estimator_out
            boxes_to_lds(img_boxes, nbox, s_part, ctx.tag, p->err, early, true);
            if (pre_w) {
                s_wup[tid_d] = wup_r;
                s_wdn[tid_d] = wdn_r;
            }
            __syncthreads();
            if (means) {  // the mailboxes hold the means themselves
                for (int k = tid_d; k < p->Ca; k += kThreads) s_g[k] = s_part[k];
            } else {
                sum_staged(s_part, p->ptiles, p->Ca, 0, p->hw, s_g);
            }
            __syncthreads();
            if (p->hidden > 0) {
                for (int m = tid_d; m < p->hidden; m += kThreads)
                    s_t[m] = gelu_erf(pre_w ? dot_row_lds(s_wdn + m * p->Ca, s_g, p->Ca, bdn_r)
                                            : dot_row(p->w_down + (size_t)m * p->Ca, s_g, p->Ca,
                                                      p->b_down ? p->b_down[m] : 0.f));
                __syncthreads();
            }
        }
        if (tid_d < 9) {
            float d;
            if (direct)
                d = pre_w ? dot_row_lds(s_wup + tid_d * Kin, p->hidden > 0 ? s_t : s_g, Kin, bup_r)
                          : estimator_out(p, wd.c * 9 + tid_d, s_g, s_t);
            else if (from_boxes)  // asked for near the end of the tap loop; otherwise wait now
                d = G::UNROLL && (uint32_t)(early[0] >> 32) == ctx.tag
                        ? __uint_as_float((uint32_t)early[0])
                        : box_get(p->dk_box + dk_idx + tid_d, ctx.tag, p->err);
            else
                d = p->dk_in[dk_idx + tid_d];
            s_dk[tid_d] = d;
        }
        __syncthreads();
        claim_next(p, ctx);  // the wait for the estimator is over
        float d[9];
#pragma unroll
        for (int k = 0; k < 9; ++k) d[k] = s_dk[k];
        if constexpr (kMatrix) {
            // block t of the wavefront: this lane's output row and four columns; per tile row the
            // six pixels from one before the first to one behind the last: the word in front
            // (upper half), the two words of the four pixels, the word behind (lower half)
#pragma unroll
            for (int t = 0; t < RY; ++t) {
                const int wi = (16 * ((mb0 & 3) + t) + 4 * mg4 + PH + MG::A) / 2;
#pragma unroll
                for (int i = 0; i < 3; ++i) {
                    const int row = 16 * (mb0 >> 2) + mrow + PH - 1 + i;
                    const uint32_t w0 = tile_d[MG::word(row, wi - 1)], w3 = tile_d[MG::word(row, wi + 2)];
                    const uint2 w12 = *reinterpret_cast<const uint2 *>(tile_d + MG::word(row, wi));
                    const float v[6] = {bf16_hi(w0), bf16_lo(w12.x), bf16_hi(w12.x), bf16_lo(w12.y), bf16_hi(w12.y), bf16_lo(w3)};
#pragma unroll
                    for (int j = 0; j < 3; ++j)
#pragma unroll
                        for (int q = 0; q < 4; ++q) acc[t][q] = fmaf(d[i * 3 + j], v[j + q], acc[t][q]);
                }
            }
        }
#pragma unroll
        for (int r = 0; r < (kMatrix ? 0 : RY + 2); ++r) {
            float v[6];
            {
                const float *src = trow_d + (r + PH - 1) * PITCH + (PH - 1);
#pragma unroll
                for (int k = 0; k < 6; ++k) v[k] = src[k];
            }
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

    if (p->dk_mode == kDkNone) claim_next(p, ctx);
    // (only in the kernel flavour that calls with such a constant are sent to: the flavour
    // the short forward calls use stays free of it)
    if (ADD && p->out_add != nullptr) {  // block-uniform
        const float add = p->out_add[wd.nc];
#pragma unroll
        for (int oy = 0; oy < RY; ++oy)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[oy][q] += add;
    }
    if constexpr (kMatrix) {
        // rounded once, through LDS (MatrixGeom::OP), then rows ty*RY ... of the tile, four
        // columns per thread, as on the other path
        if (p->dk_mode == kDkNone) __syncthreads();  // (the other modes have passed a barrier since the tap loop)
        uint32_t *otile = tbl_d;
#pragma unroll
        for (int t = 0; t < RY; ++t) {
            uint2 w;
            w.x = f32_pack2_bf16(acc[t][0], acc[t][1]);
            w.y = f32_pack2_bf16(acc[t][2], acc[t][3]);
            *reinterpret_cast<uint2 *>(otile + (16 * (mb0 >> 2) + mrow) * MG::OP + 8 * ((mb0 & 3) + t) + 2 * mg4) = w;
        }
        __syncthreads();
        const int gx = wd.x0 + 4 * tx_d;
#pragma unroll
        for (int oy = 0; oy < RY; ++oy) {
            const int gy = wd.y0 + ty_d * RY + oy;
            const uint2 w = *reinterpret_cast<const uint2 *>(otile + (ty_d * RY + oy) * MG::OP + 2 * tx_d);
            if (gy >= H) continue;
            uint16_t *dst = reinterpret_cast<uint16_t *>(op) + (size_t)gy * W + gx;
            if (p->conv_vec_ok && gx + 3 < W) {
                typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
                __builtin_nontemporal_store(u32x2{w.x, w.y}, reinterpret_cast<u32x2 *>(dst));
            } else {
                if (gx + 0 < W) dst[0] = (uint16_t)w.x;
                if (gx + 1 < W) dst[1] = (uint16_t)(w.x >> 16);
                if (gx + 2 < W) dst[2] = (uint16_t)w.y;
                if (gx + 3 < W) dst[3] = (uint16_t)(w.y >> 16);
            }
        }
        return ctx;
    }
#pragma unroll
    for (int oy = 0; oy < RY; ++oy) {
        const int gx = wd.x0 + 4 * tx_d;
        const int gy = wd.y0 + ty_d * RY + oy;
        if (gy >= H) continue;
        T *dst = op + (size_t)gy * W + gx;
        if (p->conv_vec_ok && gx + 3 < W) {
            store4(dst, acc[oy]);
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (gx + q < W) store1(dst + q, acc[oy][q]);
        }
    }
    return ctx;
}

// ---------------------------------------------------------------------------
// copy item (Eq. 4 lines 1 and 4): copy_chunk bytes of one image's identity
// channels with 16-byte non-temporal accesses when both sides allow it: 16 KiB pieces,
// two in flight - or, in the gentle mode, one access per thread at a time.
// ---------------------------------------------------------------------------
__device__ __forceinline__ Ctx copy_item(ParamsPtr p, Ctx ctx, unsigned item)
{
    const unsigned n = fdiv(item, p->div_chunks.mul, p->div_chunks.shift);
    const size_t chunk = (size_t)(item - n * p->div_chunks.d);
    // (what the conv items carry inside their tap loops comes first in the range)
    const char *src = (const char *)p->x + (size_t)n * p->img_bytes + p->idt_off + p->copy_off;
    char *dst = (char *)p->out + (size_t)n * p->img_bytes + p->idt_off + p->copy_off;
    const size_t len = p->idt_len - p->copy_off;
    const size_t begin = chunk * p->copy_chunk;
    const size_t end = begin + p->copy_chunk < len ? begin + p->copy_chunk : len;
    const int eb = p->elem_bytes;
    if (p->copy_vec_ok) {
        // Whole pieces move without a condition per access (a guarded load ends up in a basic
        // block of its own and the compiler then waits for each before the next is issued),
        // the next piece's loads going out before this piece's stores.
        const size_t nfull = (end - begin) / kCopyPiece;
        const size_t rest = begin + nfull * kCopyPiece;  // start of the partial piece, if any
        const size_t lane_off = (size_t)opaque_tid() * 16;
        if (p->copy_gentle) {
            // one access per thread in flight
            const size_t nvec = (end - begin) / (kThreads * 16);
            for (size_t i = 0; i < nvec; ++i) {
                const size_t o = begin + i * kThreads * 16 + lane_off;
                const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + o));
                if (i + 1 == nvec && begin + nvec * kThreads * 16 >= end) announce_leave(p, ctx);
                __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(dst + o));
            }
            const size_t o = begin + nvec * kThreads * 16 + lane_off;
            if (begin + nvec * kThreads * 16 < end) {
                u32x4 v = {};
                if (o + 16 <= end) v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + o));
                announce_leave(p, ctx);
                if (o + 16 <= end) __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(dst + o));
            }
        } else if (nfull > 0) {
            u32x4 v[kCopyVecPerThread], w[kCopyVecPerThread];
            auto fetch = [&](u32x4 *r, size_t i) {
#pragma unroll
                for (int k = 0; k < kCopyVecPerThread; ++k)
                    r[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(
                        src + begin + i * kCopyPiece + (size_t)k * kThreads * 16 + lane_off));
            };
            auto put = [&](const u32x4 *r, size_t i) {
#pragma unroll
                for (int k = 0; k < kCopyVecPerThread; ++k)
                    __builtin_nontemporal_store(r[k], reinterpret_cast<u32x4 *>(
                        dst + begin + i * kCopyPiece + (size_t)k * kThreads * 16 + lane_off));
            };
            // two pieces per trip, the register sets swapping roles (copying one set into the
            // other would wait for its loads on the spot)
            fetch(v, 0);
            for (size_t i = 0;; i += 2) {
                if (i + 1 < nfull)
                    fetch(w, i + 1);
                else if (rest >= end)
                    announce_leave(p, ctx);  // the item's last loads are out
                put(v, i);
                if (i + 1 >= nfull) break;
                if (i + 2 < nfull)
                    fetch(v, i + 2);
                else if (rest >= end)
                    announce_leave(p, ctx);
                put(w, i + 1);
                if (i + 2 >= nfull) break;
            }
        }
        if (!p->copy_gentle && rest < end) {  // at most one partial piece per call and image
            u32x4 v[kCopyVecPerThread];
#pragma unroll
            for (int k = 0; k < kCopyVecPerThread; ++k) {
                const size_t o = rest + (size_t)k * kThreads * 16 + lane_off;
                if (o + 16 <= end) v[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + o));
            }
            announce_leave(p, ctx);
#pragma unroll
            for (int k = 0; k < kCopyVecPerThread; ++k) {
                const size_t o = rest + (size_t)k * kThreads * 16 + lane_off;
                if (o + 16 <= end) __builtin_nontemporal_store(v[k], reinterpret_cast<u32x4 *>(dst + o));
            }
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
    return ctx;
}

// ---------------------------------------------------------------------------
// the one kernel.  KS == 0 builds the variant without conv items (used by
// esc_dynkernel_gen and for C_a == 0).
// ---------------------------------------------------------------------------
template <int KS, int RY, typename T, bool STAGED = false>
__global__ __launch_bounds__(kThreads, kBlocksPerCu) void forward_kernel(const FwdParams params)
{
    // the item functions (all inlined here) read the parameters from the kernel argument
    // segment, which starts with `params`, where they need them
    (void)params;
    ParamsPtr p = (ParamsPtr)__builtin_amdgcn_kernarg_segment_ptr();
    __builtin_amdgcn_s_setprio(kPrioHigh);

    // Blocks are handed to the chip's eight dies (XCDs, each with its own L2) round robin
    // by block index.  Each die gets one contiguous eighth of every kind of item, so that
    // neighbouring tiles - and the pool tiles over the same pixels - meet in one L2; inside
    // a die, block number `slot` takes entries slot, slot + S, ... of the die's list.
    const unsigned die = blockIdx.x % kXcds, slot = blockIdx.x / kXcds, S = gridDim.x / kXcds;
    unsigned pool_base, pool_cnt, gen_base, gen_cnt, conv_base, conv_cnt, copy_base, copy_cnt;
    die_share(p->n_pool, die, pool_base, pool_cnt);
    die_share(p->n_gen, die, gen_base, gen_cnt);
    die_share(p->n_conv, die, conv_base, conv_cnt);
    die_share(p->n_copy, die, copy_base, copy_cnt);
    // conv and copy entries alternate in groups of mix_a + mix_b while both last
    const unsigned group = p->mix_a + p->mix_b;
    unsigned groups = 0;
    if (conv_cnt > 0 && copy_cnt > 0) {
        const unsigned ga = fdiv(conv_cnt, p->div_mix_a.mul, p->div_mix_a.shift), gb = fdiv(copy_cnt, p->div_mix_b.mul, p->div_mix_b.shift);
        groups = ga < gb ? ga : gb;
    }
    const unsigned first_mixed = pool_cnt + gen_cnt;
    const unsigned total = first_mixed + conv_cnt + copy_cnt;
    Ctx ctx;
    ctx.tag = 0;
    ctx.have_tag = false;
    ctx.last_item = false;
    ctx.announced = false;
    ctx.left = 0;
    ctx.claim = 0;
    // Which entries a block processes.  A call that fits into one round of resident blocks:
    // entry `slot` (and slot + S, ... if any).  Longer calls: the items differ too much in
    // duration for a fixed deal, so the die's list is dealt to its eight block groups
    // (entries k, k + 8, ... to group k = slot % 8) and inside a group each block starts
    // with the entry of its rank and takes every further one from the group's queue - one
    // atomic per item (see claim_next), looked at when the item ends.
    const bool dynamic = p->dynamic != 0;
    const unsigned k8 = slot % kXcds, rank = slot / kXcds, members8 = (S - k8 + kXcds - 1) / kXcds;
    unsigned turn = 0;
    for (unsigned li = dynamic ? k8 + kXcds * rank : slot; li < total;) {
        // kind and index of this entry
        int kind;  // 0 pool, 1 gen, 2 conv, 3 copy
        unsigned idx;
        if (li < pool_cnt) {
            kind = 0;
            idx = pool_base + li;
        } else if (li < first_mixed) {
            kind = 1;
            idx = gen_base + (li - pool_cnt);
        } else {
            const unsigned j = li - first_mixed;
            bool is_conv;
            unsigned local;
            if (j < groups * group) {
                const unsigned g = fdiv(j, p->div_mix.mul, p->div_mix.shift), r = j - g * group;
                is_conv = r < p->mix_a;
                local = is_conv ? g * p->mix_a + r : g * p->mix_b + (r - p->mix_a);
            } else {
                const unsigned jj = j - groups * group;
                const unsigned conv_left = conv_cnt - groups * p->mix_a;
                is_conv = jj < conv_left;
                local = is_conv ? groups * p->mix_a + jj : groups * p->mix_b + (jj - conv_left);
            }
            kind = is_conv ? 2 : 3;
            idx = (is_conv ? conv_base : copy_base) + local;
        }
        ctx.last_item = !dynamic && li + S >= total;
        if (kind == 0 || kind == 3) claim_next(p, ctx);
        if (kind == 0) {
            ctx = pool_item<T>(p, ctx, idx);
        } else if (kind == 1) {
            if constexpr (STAGED) {
                // the gsum items of every (image, channel), then one gen item per image
                const unsigned n_gsum = p->n_gsum;
                if (idx < n_gsum)
                    ctx = gsum_item(p, ctx, idx);
                else
                    ctx = gen_item_staged(p, ctx, idx - n_gsum, n_gsum > 0);
            } else {
                ctx = gen_item(p, ctx, idx);
            }
        } else if (kind == 2) {
            if constexpr (KS > 0)
                ctx = conv_item<KS, RY, T, STAGED>(p, ctx, idx);
        } else {
            if (KS == 0 && p->aux_n > 0) {
                if constexpr (KS == 0) {
                    const int e = (int)idx * kThreads + (int)threadIdx.x;
                    if (e < p->aux_n) dense_table_entry(p->aux_lk, p->aux_Ca, p->aux_Ks, p->aux_Kse, p->aux_nw, p->aux_wa, e);
                }
            } else {
                ctx = copy_item(p, ctx, idx);
            }
        }
        if (dynamic) {
            if (threadIdx.x == kThreads - 1) g_next[turn & 1] = k8 + kXcds * (members8 + ctx.claim);
            __syncthreads();  // also: LDS is reused by the next item
            li = g_next[turn & 1];
            ++turn;
        } else {
            __syncthreads();  // LDS is reused by the next item
            li += S;
        }
    }
    // A block without items still belongs to its group.  The last block of a group to have
    // announced its leave opens the next call for the group: leave counter back to zero, tag + 1.
    ctx.last_item = true;
    announce_leave(p, ctx);
    if (threadIdx.x == kThreads - 1) {
        const unsigned g = blockIdx.x % kGroups;
        const unsigned members = (gridDim.x - g + kGroups - 1) / kGroups;
        if (ctx.left == members - 1) {
            __hip_atomic_store(p->queue + g * kCtlStride, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(p->done + g * kCtlStride, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(p->epoch + g * kCtlStride, ctx.tag + 1u == 0u ? 1u : ctx.tag + 1u, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}


}  // namespace
}  // namespace esc

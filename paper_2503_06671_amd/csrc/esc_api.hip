// Host side of the ConvAttn forward library for gfx950 (MI355X): argument checks, the
// layout of the workspace, the plan that cuts a call into work items, and the C ABI
// declared in include/esc_convattn.h.  The kernels live in esc_kernels.hpp and are
// instantiated per kernel size in esc_variants.hip.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "esc_kernels.hpp"
#include "esc_backward.hpp"
#include "esc_dense.hpp"
#include "esc_ffn.hpp"
#include "esc_pointwise.hpp"

namespace esc {

// one pair per kernel size, defined in esc_variants.hip (-DESC_KS=<Ks>)
#define ESC_DECL_KS(K)                                                                                    \
    hipError_t launch_ks_##K(int ry, bool bf16, bool staged, unsigned grid, hipStream_t s, const FwdParams &p); \
    hipError_t occupancy_ks_##K(int ry, bool bf16, bool staged, int *blocks_per_cu);
#define ESC_FOR_EACH_KS(X) X(0) X(1) X(3) X(5) X(7) X(9) X(11) X(13) X(15) X(17) X(19) X(21) X(23) X(25) X(27) X(29) X(31)
ESC_FOR_EACH_KS(ESC_DECL_KS)
#undef ESC_DECL_KS

}  // namespace esc

namespace {

using namespace esc;

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
    int ptiles_x, ptiles;
    size_t ctl_off, pool_off, dk_off, g_off, total;
};

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

bool ws_layout(int N, int Ca, int H, int W, WsLayout *l)
{
    if (N < 1 || Ca < 0 || H < 1 || W < 1) return false;
    const size_t hw = (size_t)H * (size_t)W;
    if (hw >= ((size_t)1 << 31)) return false;
    l->ptiles_x = (W + kPoolTileW - 1) / kPoolTileW;
    l->ptiles = l->ptiles_x * ((H + kPoolTileH - 1) / kPoolTileH);
    size_t off = 0;
    l->ctl_off = off;
    off = round_up(off + kCtlWords * sizeof(uint32_t), kWsAlign);
    l->pool_off = off;
    off = round_up(off + (size_t)N * Ca * l->ptiles * sizeof(u64), kWsAlign);
    l->dk_off = off;
    off = round_up(off + (size_t)N * Ca * 9 * sizeof(u64), kWsAlign);
    l->g_off = off;
    off = round_up(off + (size_t)N * Ca * sizeof(u64), kWsAlign);
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

// do the byte ranges [a, a + na) and [b, b + nb) share a byte?
bool overlaps(const void *a, size_t na, const void *b, size_t nb)
{
    const uintptr_t ua = (uintptr_t)a, ub = (uintptr_t)b;
    return na > 0 && nb > 0 && ua < ub + nb && ub < ua + na;
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


// compute units of the current device (asked once per device)
int device_cus()
{
    constexpr int kMaxDev = 64;
    static int cus[kMaxDev];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) return 0;
    if (cus[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) n = 0;
        cus[dev] = n;
    }
    return cus[dev];
}

// Lays the items out for the grid: how many blocks per die, whether the conv items can
// pool for themselves, how big a copy item is and how conv and copy items alternate.
// n_conv, n_gen and the pass-through range are set; n_pool holds the pool-item count that
// applies if pooling is not fused.
struct Plan {
    unsigned per_die;
};

Plan plan_items(FwdParams &p, int Ks, int blocks_per_cu, int carry_grains)
{
    const unsigned U = (unsigned)device_cus() / kXcds;          // compute units per die
    const unsigned Smax = (unsigned)blocks_per_cu * (U ? U : 1);  // resident blocks per die
    auto per_die_of = [](u64 n) { return (unsigned)((n + kXcds - 1) / kXcds); };

    // Few pool tiles per image: one gen item per image runs the estimator while the conv
    // items multiply, and they pick DK up on the way (asked for inside the tap loop) - if the
    // gen items still fit beside all conv items (fused pooling).  Otherwise the conv items
    // run the estimator themselves (direct mode).  Measured at 180 x 320, the hop is the
    // faster of the two for every Ks.
    if (p.pool_mode == kPoolItems && p.dk_mode == kDkDirect && p.n_conv > 0 &&
        per_die_of(p.n_conv) + per_die_of((u64)p.N) <= Smax) {
        p.dk_mode = kDkBoxes;
        p.n_gen = (unsigned)p.N;
    }

    // all conv items (and the gen items they wait for) in the first round => fused pooling
    const bool one_round = p.n_conv > 0 && per_die_of(p.n_conv) + per_die_of(p.n_gen) <= Smax;
    if (p.pool_mode == kPoolItems && one_round) {
        p.pool_mode = kPoolFused;
        p.n_pool = 0;
    } else if (p.dk_mode == kDkMeans) {
        // Longer calls: a conv item that runs the estimator itself pays for it (mailboxes,
        // barriers) in every one of a block's items, while the hop it saves is waited for once
        // per call: one gen item per image publishes DK instead (measured at 540 x 960).
        p.n_gen = p.n_gsum + (unsigned)p.N;
        p.dk_mode = kDkBoxes;
    }

    // Short calls (the conv items' own chain of tile load, taps, estimator and store is most of
    // them) copy gently: the blocks left over beside the resident conv items get through the
    // pass-through range in about a dozen accesses per thread, one in flight at a time.
    {
        const u64 others0 = (u64)p.n_pool + p.n_gen + p.n_conv, resident0 = (u64)kXcds * Smax;
        const u64 spare = resident0 > others0 + kXcds * 4 ? resident0 - others0 - kXcds * 3 : 0;
        // (calls without an estimator - DK given, or none - take the same arrangement when their conv items fit)
        const bool resident_convs = p.pool_mode == kPoolFused || (p.pool_mode == kPoolNone && one_round);
        p.copy_gentle = resident_convs && p.n_gsum == 0 &&
                        (p.dk_mode == kDkDirect || p.dk_mode == kDkBoxes || p.dk_mode == kDkGiven || p.dk_mode == kDkNone) &&
                        (u64)p.N * p.idt_len <= spare * 12 * (u64)kThreads * 16;
    }

    // Carried copy, everywhere else: every conv item moves an equal share of its image's
    // pass-through range, in 4 KiB grains, as many as its registers hold; copy items are left
    // with what lies beyond.
    p.carry_g = 0;
    p.copy_off = 0;
    if (carry_grains > 0 && !p.copy_gentle && p.n_conv > 0 && p.idt_len > 0 && p.copy_vec_ok) {
        const size_t per_img = p.n_conv / (size_t)p.N;
        const size_t grains = (p.idt_len + kGrain - 1) / kGrain;
        size_t g = (grains + per_img - 1) / per_img;
        if (g > (size_t)carry_grains) g = (size_t)carry_grains;
        p.carry_g = (unsigned)g;
        const size_t carried = per_img * g * kGrain;
        p.copy_off = carried < p.idt_len ? carried : p.idt_len;
    }
    const size_t rest_len = p.idt_len - p.copy_off;  // pass-through bytes per image left to copy items

    // rough time shares of the arithmetic and of the pass-through traffic decide how many
    // copy items there are to a conv item (and with that how small they are): 1, 2 or 3,
    // thresholds from sweeps at 540 x 960 with Ks = 7 ... 31
    const double pix = (double)p.N * p.Ca * p.H * p.W;
    const double t_valu = 2.0 * Ks * Ks * pix / 50e12;  // what a conv item sustains, its loads included
    const double t_copy = 2.0 * (double)p.N * (double)rest_len / 4.5e12;
    unsigned a = 1, b = 1;
    if (t_valu > 0 && t_copy > 0) {
        const double share = t_valu / (t_valu + t_copy);
        if (share < 0.6) b = 2;
        if (share < 0.3) b = 3;
    }

    // copy items: as many as the pattern pairs with the conv items; if the whole call fits
    // into one round of resident blocks, as many as still fit
    p.n_copy = 0;
    p.copy_chunk = kCopyPiece;
    if (rest_len > 0) {
        u64 want = p.n_conv > 0 ? (u64)p.n_conv * b / a : (u64)kXcds * Smax * 4;
        const u64 others = (u64)p.n_pool + p.n_gen + p.n_conv;
        const u64 resident = (u64)kXcds * Smax;
        if (others + kXcds * 4 < resident && others + want > resident && (resident - others) * 4 >= want)
            want = resident - others - kXcds * 3;  // the lists are rounded up per kind and die
        // gentle copying moves one access per thread at a time: as many items as fit, cut finely
        const size_t grain = p.copy_gentle ? (size_t)kThreads * 16 : kCopyPiece;
        if (p.copy_gentle && others + kXcds * 4 < resident) want = resident - others - kXcds * 3;
        // fused pooling without room beside the conv items: the copy comes after them, and
        // every block should get a share of it
        if (p.pool_mode == kPoolFused && !p.copy_gentle && want < 2 * resident) want = 2 * resident;
        if (want < 1) want = 1;
        u64 per_img = (want + p.N / 2) / p.N;
        if (per_img < 1) per_img = 1;
        size_t chunk = (rest_len + per_img - 1) / per_img;
        chunk = (chunk + grain - 1) / grain * grain;
        const size_t chunks = (rest_len + chunk - 1) / chunk;
        p.copy_chunk = chunk;
        p.div_chunks = make_div((uint32_t)chunks);
        p.n_copy = (unsigned)(chunks * p.N);
    }

    // (the estimator launch of a dense call: its copy entries build the dense kernel's table)
    if (p.aux_n > 0 && p.n_conv == 0 && rest_len == 0) p.n_copy = (unsigned)((p.aux_n + kThreads - 1) / kThreads);

    // Alternation in layers, so that consecutive blocks - which the dispatcher spreads over a
    // die's compute units - are of one kind and every unit gets every kind: U conv entries,
    // then copy entries in proportion to what there is of each kind - times 3/4, so that the
    // conv entries (the long ones) run out first and the list ends with copy entries, which
    // even out the end of the call (measured at 540 x 960: 2 - 3 % over plain proportion for
    // Ks = 7 ... 17, and over the fixed 1:1 / 1:2 / 1:3 patterns before it).
    if (p.pool_mode == kPoolFused || p.copy_gentle) {
        p.mix_a = p.mix_b = 1u << 30;  // all conv items first: they must all be in the first round
    } else {
        const unsigned Ul = U ? U : 1;
        p.mix_a = Ul;
        p.mix_b = Ul;
        if (p.n_conv > 0 && p.n_copy > 0) {
            const double share = 0.75 * (double)p.n_copy / (double)p.n_conv;
            const double mb = share * Ul + 0.5;
            p.mix_b = mb < 1.0 ? 1u : mb > 64.0 * Ul ? 64u * Ul : (unsigned)mb;
        }
    }
    p.div_mix = make_div(p.mix_a + p.mix_b);
    p.div_mix_a = make_div(p.mix_a);
    p.div_mix_b = make_div(p.mix_b);

    Plan plan;
    unsigned need = per_die_of(p.n_pool) + per_die_of(p.n_gen) + per_die_of(p.n_conv) + per_die_of(p.n_copy);
    plan.per_die = need < Smax ? need : Smax;
    p.dynamic = need > Smax;
    if (plan.per_die < (unsigned)kGroups / kXcds) plan.per_die = kGroups / kXcds;  // every block group needs a member
    return plan;
}

// index of a kernel size in the variant tables: 0 for the variant without conv items,
// (Ks + 1) / 2 for odd Ks
typedef hipError_t (*LaunchFn)(int, bool, bool, unsigned, hipStream_t, const FwdParams &);
typedef hipError_t (*OccupancyFn)(int, bool, bool, int *);
constexpr int kKsSlots = 17;
#define ESC_LAUNCH_ENTRY(K) launch_ks_##K,
#define ESC_OCC_ENTRY(K) occupancy_ks_##K,
const LaunchFn kLaunch[kKsSlots] = {ESC_FOR_EACH_KS(ESC_LAUNCH_ENTRY)};
const OccupancyFn kOccupancy[kKsSlots] = {ESC_FOR_EACH_KS(ESC_OCC_ENTRY)};
#undef ESC_LAUNCH_ENTRY
#undef ESC_OCC_ENTRY

// Resident blocks per compute unit the grid of a variant may count on: what the runtime's
// occupancy query grants on the device in hand, asked once per device and variant, capped
// at what the kernel is compiled for.  0 = the variant cannot run here.
int resident_blocks_per_cu(int ks_slot, int ry, bool bf16, bool staged)
{
    constexpr int kMaxDev = 64;
    static signed char cache[kMaxDev][kKsSlots][2][2][2];  // 0 = not asked yet, else answer + 1
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) return 0;
    signed char &slot = cache[dev][ks_slot][ry == 4][bf16][staged];
    if (slot == 0) {
        int n = 0;
        if (kOccupancy[ks_slot](ry, bf16, staged, &n) != hipSuccess) n = 0;
        if (n > kBlocksPerCu) n = kBlocksPerCu;
        if (n < 0) n = 0;
        slot = (signed char)(n + 1);
    }
    return slot - 1;
}

// Picks the register blocking, plans the items and launches the one kernel of a call.
esc_status launch_forward(FwdParams &p, int Ks, bool bf16, hipStream_t s)
{
    const int cus = device_cus();
    if (cus < (int)kXcds) return ESC_ERR_HIP;
    int ry = 2;
    if (Ks > 0) {
        // taller register blocks (fewer halo rows, more arithmetic per item's fixed latencies)
        // once they still give every compute unit two tiles
        const size_t tiles4 = (size_t)((p.W + kTileW - 1) / kTileW) * ((p.H + 63) / 64) * p.N * p.Ca;
        ry = (tiles4 >= 2 * (size_t)cus && Ks <= 17) ? 4 : 2;
        const int th = 16 * ry;
        const int tiles_x = (p.W + kTileW - 1) / kTileW;
        const int tiles_y = (p.H + th - 1) / th;
        p.div_tiles_x = make_div((uint32_t)tiles_x);
        p.div_tiles_y = make_div((uint32_t)tiles_y);
        const size_t n_conv = (size_t)tiles_x * tiles_y * p.N * p.Ca;
        if (n_conv >= ((size_t)1 << 30)) return ESC_ERR_UNSUPPORTED;
        p.n_conv = (unsigned)n_conv;
    }
    const u64 total = (u64)p.n_pool + p.n_gen + p.n_conv + (p.idt_len > 0 ? 1 : 0);
    if (total == 0) return ESC_OK;
    // the blocks of the grid wait for one another, so all of them must be resident at once:
    // the grid is sized by what the runtime says fits on this device
    const int ks_slot = (Ks + 1) / 2;
    const int bpc = resident_blocks_per_cu(ks_slot, ry, bf16, p.staged != 0);
    if (bpc < 1) return ESC_ERR_UNSUPPORTED;
    const Plan plan = plan_items(p, Ks, bpc, Ks > 0 ? conv_carry_grains(Ks, ry, bf16) : 0);
    if ((u64)p.n_pool + p.n_gen + p.n_conv + p.n_copy >= ((u64)1 << 30)) return ESC_ERR_UNSUPPORTED;
    const unsigned grid = plan.per_die * kXcds;
    return kLaunch[ks_slot](ry, bf16, p.staged != 0, grid, s, p) == hipSuccess ? ESC_OK : ESC_ERR_HIP;
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
    p.ptiles_x = l.ptiles_x;
    p.ptiles = l.ptiles;
    p.hw = (float)((double)H * (double)W);
    p.elem_bytes = dt == ESC_F32 ? 4 : 2;
    p.div_ptiles = make_div((uint32_t)l.ptiles);
    p.div_ptiles_x = make_div((uint32_t)l.ptiles_x);
    // aligned 4-element chunk loads (halo tile, pool tile) need W % 4 == 0 and an aligned base
    p.conv_ld_vec = (W % 4 == 0) && ((uintptr_t)x % (4 * (size_t)p.elem_bytes) == 0);
    // bf16: 16-byte pieces of 8 elements where the width and the base allow them
    if (p.conv_ld_vec && dt == ESC_BF16 && W % 8 == 0 && (uintptr_t)x % 16 == 0) p.conv_ld_vec = 2;
    p.div_ca = make_div((uint32_t)(Ca > 0 ? Ca : 1));
    p.div_tiles_x = p.div_tiles_y = p.div_chunks = p.div_mix = p.div_mix_a = p.div_mix_b = make_div(1);
    if (gen != nullptr && Ca > 0) {
        p.dk_mode = ((size_t)Ca * l.ptiles <= (size_t)kDirectMaxBoxes) ? kDkDirect : kDkFromG;
        p.pool_mode = kPoolItems;
        p.hidden = gen->hidden;
        p.w_down = gen->w_down;
        p.b_down = gen->b_down;
        p.w_up = gen->w_up;
        p.b_up = gen->b_up;
        const size_t n_pool = (size_t)N * Ca * l.ptiles;
        if (n_pool >= ((size_t)1 << 30)) return ESC_ERR_UNSUPPORTED;
        p.n_pool_tiles = (unsigned)n_pool;
        p.n_pool = (unsigned)((n_pool + kPoolBatch - 1) / kPoolBatch);
        // Larger planes: a gsum item per (image, channel), then a gen item per image that turns
        // the means into DK; the conv items pick DK up as from any gen item.  These calls, and
        // calls whose estimator is beyond the small ones that gen_item prefetches, run the
        // kernel flavour with the staged estimator items.
        const int K = gen->hidden > 0 ? gen->hidden : Ca;
        const bool small_est = K <= 16 && Ca <= 16 && gen->hidden <= kThreads;
        p.staged = p.dk_mode == kDkFromG || !small_est;
        if (p.dk_mode == kDkFromG) {
            p.n_gsum = (unsigned)((size_t)N * Ca);
            if (small_est) {  // the conv items run the estimator themselves, from the means
                p.n_gen = p.n_gsum;
                p.dk_mode = kDkMeans;
            } else {
                p.n_gen = p.n_gsum + (unsigned)N;
                p.dk_mode = kDkBoxes;
            }
        }
    }
    char *w = (char *)workspace;
    p.err = (unsigned *)(w + l.ctl_off) + kCtlErrWord;
    p.epoch = (unsigned *)(w + l.ctl_off) + kCtlEpochWord;
    p.done = (unsigned *)(w + l.ctl_off) + kCtlDoneWord;
    p.queue = (unsigned *)(w + l.ctl_off) + kCtlQueueWord;
    p.pool_box = (u64 *)(w + l.pool_off);
    p.dk_box = (u64 *)(w + l.dk_off);
    p.g_box = (u64 *)(w + l.g_off);
    return ESC_OK;
}

// Eq. 4 line 2 alone on checked arguments: one launch of the variant without conv items.
// dense_lk / dense_table: the dense kernel's A-operand table (dense_table_entry) is built by the
// same launch, beside the pooling, from the Ks x Ks x C_a x C_a kernel dense_lk (nullptr: not)
esc_status enqueue_dynkernel(const void *x, esc_dtype dt, int N, int C, int H, int W, int C_a, const esc_gen_params *gen,
                             float *dk_out, void *workspace, const WsLayout &l, hipStream_t stream,
                             const float *dense_lk = nullptr, int dense_ks = 0, uint32_t *dense_table = nullptr)
{
    FwdParams p;
    esc_status st = setup_common(p, x, dt, N, C, H, W, C_a, gen, workspace, l);
    if (st != ESC_OK) return st;
    if (dense_lk != nullptr) {
        p.aux_lk = dense_lk;
        p.aux_wa = dense_table;
        p.aux_Ca = C_a;
        p.aux_Ks = dense_ks;
        p.aux_Kse = dense_effective_ks(dense_ks);
        p.aux_nw = dt == ESC_BF16 ? 2 : 3;
        p.aux_n = dense_table_entries(p.aux_Kse);
    }
    p.dk_out = dk_out;
    p.dk_mode = kDkBoxes;  // no conv items here: gen items write dk_out, each from its image's pool sums
    p.n_gen = (unsigned)N;
    p.n_gsum = 0;
    return launch_forward(p, 0, dt == ESC_BF16, stream);
}

// The forward on checked arguments: one launch.  `out` holds out_c channels per image, of
// which the first C_a are written by the conv items; with_copy adds the pass-through copy
// of channels C_a .. C (then out_c == C).  out_add: a constant per (image, channel) for the
// conv items to add to their plane's outputs, or NULL.
esc_status enqueue_forward(const void *x, esc_dtype dt, int N, int C, int H, int W, int C_a, const float *lk, int Ks,
                           long lk_channel_stride, const esc_gen_params *gen, const float *dk_in, void *out, int out_c,
                           bool with_copy, void *workspace, const WsLayout &l, hipStream_t stream,
                           const float *out_add = nullptr)
{
    const size_t es = dt == ESC_F32 ? 4 : 2;
    const uintptr_t xa = (uintptr_t)x, oa = (uintptr_t)out;
    FwdParams p;
    esc_status st = setup_common(p, x, dt, N, C, H, W, C_a, gen, workspace, l);
    if (st != ESC_OK) return st;
    p.out = out;
    p.out_c = out_c;
    p.lk = lk;
    p.lk_cstride = lk_channel_stride;
    p.dk_in = (gen == nullptr && C_a > 0) ? dk_in : nullptr;
    if (p.dk_in != nullptr) p.dk_mode = kDkGiven;
    p.out_add = C_a > 0 ? out_add : nullptr;
    if (p.out_add != nullptr) p.staged = 1;  // the kernel flavour whose conv items know of it
    // 16-byte (fp32) / 8-byte (bf16) row stores need W % 4 == 0 and an aligned base
    p.conv_vec_ok = (W % 4 == 0) && (oa % (4 * es) == 0);
    if (with_copy && C_a < C) {
        const size_t plane = (size_t)H * W * es;
        p.img_bytes = plane * C;
        p.idt_off = plane * C_a;
        p.idt_len = plane * (C - C_a);
        p.copy_vec_ok = (xa % 16 == 0) && (oa % 16 == 0) && (p.img_bytes % 16 == 0) && (p.idt_off % 16 == 0);
    }
    const int ks_variant = C_a > 0 ? Ks : 0;
    return launch_forward(p, ks_variant, dt == ESC_BF16, stream);
}

// Workspace of esc_convattn_fused_forward: the forward's own workspace first, then F_res
// [N,C_a,H,W] in the storage type and, with LK^c, F_att (*) LK^c (same shape) and DK.
struct FusedLayout {
    WsLayout ws;
    size_t fres_off, pw_off, dk_off, total;
};

bool fused_layout(int N, int Ca, int H, int W, esc_dtype dt, bool with_lkc, FusedLayout *f)
{
    if (dt != ESC_F32 && dt != ESC_BF16) return false;
    if (!ws_layout(N, Ca, H, W, &f->ws)) return false;
    const size_t es = dt == ESC_F32 ? 4 : 2;
    const size_t slice = round_up((size_t)N * Ca * H * W * es, kWsAlign);
    size_t off = f->ws.total;
    f->fres_off = off;
    off += slice;
    f->pw_off = off;
    f->dk_off = off;
    if (with_lkc) {
        off += slice;
        f->dk_off = off;
        off += round_up((size_t)N * Ca * 9 * sizeof(float), kWsAlign);
    }
    f->total = off;
    return true;
}

// Workspace of esc_convattn_dense_forward: the forward's own workspace (the estimator
// launch uses its mailboxes), then DK [N,C_a,3,3] fp32 and the rearranged dense weights.
struct DenseLayout {
    WsLayout ws;
    size_t dk_off, wt_off, total;
};

bool dense_layout(int N, int Ca, int H, int W, int Ks, DenseLayout *d)
{
    if (Ks < 1 || !ws_layout(N, Ca, H, W, &d->ws)) return false;
    size_t off = d->ws.total;
    d->dk_off = off;
    off += round_up((size_t)N * Ca * 9 * sizeof(float), kWsAlign);
    d->wt_off = off;
    off += round_up(dense_weight_floats(Ca, Ks) * sizeof(float), kWsAlign);
    d->total = off;
    return true;
}

// Workspace of esc_convattn_backward: the forward's own workspace (the input gradient is a
// forward launch), then the fp32 pieces BackwardParams names.
struct BackwardLayout {
    WsLayout ws;
    size_t partial_off, ddk_off, g_off, t_off, du_off, dgc_off, dkf_off, lkf_off, total;
};

bool backward_layout(int N, int Ca, int H, int W, int Ks, int hidden, BackwardLayout *b)
{
    if (Ks < 1 || hidden < 0 || !ws_layout(N, Ca, H, W, &b->ws)) return false;
    size_t off = b->ws.total;
    auto take = [&](size_t floats) {
        const size_t at = off;
        off += round_up((floats > 0 ? floats : 1) * sizeof(float), kWsAlign);
        return at;
    };
    const size_t K = hidden > 0 ? (size_t)hidden : (size_t)Ca;
    b->partial_off = take(corr_partial_floats(N, Ca, H, W, Ks));
    b->ddk_off = take((size_t)N * Ca * 9);
    b->g_off = take((size_t)N * Ca);
    b->t_off = take((size_t)N * K);
    b->du_off = take((size_t)N * hidden);
    b->dgc_off = take((size_t)N * Ca);
    b->dkf_off = take((size_t)N * Ca * 9);
    b->lkf_off = take((size_t)Ca * Ks * Ks);
    b->total = off;
    return true;
}

// The mailboxes and counters of esc_convattn_forward_noalloc: one copy per device, in the
// code object's data segment, so that a call needs no allocation and no preparation.  It is
// laid out like a caller's workspace and starts out as esc_workspace_init would leave it
// (everything zero, the groups' call counters 1), by constant initialisation.
struct Scratch {
    uint32_t words[ESC_NOALLOC_SCRATCH_BYTES / sizeof(uint32_t)];
    constexpr Scratch() : words{}
    {
        for (size_t g = 0; g < (size_t)kGroups; ++g) words[kCtlEpochWord + g * kCtlStride] = 1u;
    }
};
static __device__ __align__(256) Scratch scratch;

// Device address of this device's copy of `scratch` (the name is a host-side stand-in, not
// an address a kernel could use): asked once per device, with that device current.
esc_status scratch_address(void **out_ptr)
{
    constexpr int kMaxDev = 64;
    static void *ptrs[kMaxDev];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) return ESC_ERR_HIP;
    if (ptrs[dev] == nullptr) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return ESC_ERR_HIP;
        ptrs[dev] = ptr;
    }
    *out_ptr = ptrs[dev];
    return ESC_OK;
}

// esc_convattn_forward and esc_convattn_forward_noalloc: the same checks, plan and kernel;
// they differ in where the workspace lives.
esc_status forward_impl(const void *x, esc_dtype dt, int N, int C, int H, int W, int C_a, const float *lk, int Ks,
                        long lk_channel_stride, const esc_gen_params *gen, const float *dk_in, void *out,
                        void *workspace, size_t workspace_bytes, bool own_scratch, void *stream)
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
    if (overlaps(x, bytes, out, bytes)) return ESC_ERR_ALIAS;
    WsLayout l;
    if (!ws_layout(N, C_a, H, W, &l)) return ESC_ERR_SHAPE;
    if (own_scratch) {
        // the built-in scratch has a fixed size: larger shapes need a caller's workspace
        if (l.total > sizeof(Scratch)) return ESC_ERR_WORKSPACE;
        if ((st = scratch_address(&workspace)) != ESC_OK) return st;
        workspace_bytes = sizeof(Scratch);
    }
    if ((st = check_ws(workspace, workspace_bytes, l.total)) != ESC_OK) return st;
    if (overlaps(workspace, workspace_bytes, out, bytes) || overlaps(workspace, workspace_bytes, x, bytes))
        return ESC_ERR_ALIAS;
    if (C_a > 0) {
        const size_t lk_bytes = ((size_t)(lk_channel_stride != 0 ? C_a - 1 : 0) * (size_t)lk_channel_stride +
                                 (size_t)Ks * Ks) * sizeof(float);
        if (overlaps(lk, lk_bytes, out, bytes)) return ESC_ERR_ALIAS;
        if (gen == nullptr && dk_in != nullptr && overlaps(dk_in, (size_t)N * C_a * 9 * sizeof(float), out, bytes))
            return ESC_ERR_ALIAS;
    }

    return enqueue_forward(x, dt, N, C, H, W, C_a, lk, Ks, lk_channel_stride, gen, dk_in, out, C, true, workspace, l,
                           (hipStream_t)stream);
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
    {
        const size_t x_bytes = (size_t)N * C * H * W * (dt == ESC_F32 ? 4 : 2);
        const size_t dk_bytes = (size_t)N * C_a * 9 * sizeof(float);
        if (overlaps(dk_out, dk_bytes, x, x_bytes) || overlaps(dk_out, dk_bytes, workspace, workspace_bytes) ||
            overlaps(workspace, workspace_bytes, x, x_bytes))
            return ESC_ERR_ALIAS;
    }
    return enqueue_dynkernel(x, dt, N, C, H, W, C_a, gen, dk_out, workspace, l, (hipStream_t)stream);
}

esc_status esc_convattn_forward(const void *x, esc_dtype dt, int N, int C, int H, int W, int C_a,
                                const float *lk, int Ks, long lk_channel_stride,
                                const esc_gen_params *gen, const float *dk_in, void *out,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    return forward_impl(x, dt, N, C, H, W, C_a, lk, Ks, lk_channel_stride, gen, dk_in, out, workspace,
                        workspace_bytes, false, stream);
}

esc_status esc_convattn_forward_noalloc(const void *x, esc_dtype dt, int N, int C, int H, int W, int C_a,
                                        const float *lk, int Ks, long lk_channel_stride,
                                        const esc_gen_params *gen, const float *dk_in, void *out, void *stream)
{
    return forward_impl(x, dt, N, C, H, W, C_a, lk, Ks, lk_channel_stride, gen, dk_in, out, nullptr, 0, true,
                        stream);
}


size_t esc_fused_workspace_bytes(int N, int C_a, int H, int W, esc_dtype dt, int with_lk_c)
{
    FusedLayout f;
    if (!fused_layout(N, C_a, H, W, dt, with_lk_c != 0, &f)) return 0;
    return f.total;
}

esc_status esc_convattn_fused_forward(const void *x, esc_dtype dt, int N, int C, int H, int W, int C_a,
                                      const float *lk_c, const float *lk, int Ks, long lk_channel_stride,
                                      const esc_gen_params *gen, const float *dk_in, const float *w_fuse,
                                      const float *b_fuse, const void *residual, void *out, void *workspace,
                                      size_t workspace_bytes, void *stream)
{
    esc_status st = check_common(x, dt, N, C, H, W, C_a);
    if (st != ESC_OK) return st;
    if (out == nullptr || w_fuse == nullptr) return ESC_ERR_NULL;
    if (Ks < 1 || (Ks % 2) == 0) return Ks < 1 ? ESC_ERR_SHAPE : ESC_ERR_UNSUPPORTED;
    if (Ks > kMaxKs || C > kPointwiseMaxK) return ESC_ERR_UNSUPPORTED;
    if (C_a > 0 && lk == nullptr) return ESC_ERR_NULL;
    if (lk_channel_stride != 0 && lk_channel_stride < (long)Ks * Ks) return ESC_ERR_SHAPE;
    if (gen != nullptr && (st = check_gen(gen, C_a)) != ESC_OK) return st;
    const size_t es = dt == ESC_F32 ? 4 : 2;
    if (((uintptr_t)out % es) != 0 || ((uintptr_t)residual % es) != 0) return ESC_ERR_SHAPE;
    const size_t bytes = (size_t)N * C * H * W * es;
    if (overlaps(x, bytes, out, bytes) || (residual != nullptr && overlaps(residual, bytes, out, bytes)))
        return ESC_ERR_ALIAS;
    const bool with_lkc = lk_c != nullptr && C_a > 0;
    FusedLayout f;
    if (!fused_layout(N, C_a, H, W, dt, with_lkc, &f)) return ESC_ERR_SHAPE;
    if ((st = check_ws(workspace, workspace_bytes, f.total)) != ESC_OK) return st;
    if (overlaps(workspace, workspace_bytes, out, bytes) || overlaps(workspace, workspace_bytes, x, bytes) ||
        (residual != nullptr && overlaps(workspace, workspace_bytes, residual, bytes)))
        return ESC_ERR_ALIAS;
    if (overlaps(w_fuse, (size_t)C * C * sizeof(float), out, bytes)) return ESC_ERR_ALIAS;

    hipStream_t s = (hipStream_t)stream;
    const bool bf16 = dt == ESC_BF16;
    const size_t plane = (size_t)H * W;
    char *w = (char *)workspace;
    void *fres = w + f.fres_off;
    if (C_a > 0) {
        const void *conv_in = x;
        int conv_c = C;
        const esc_gen_params *conv_gen = gen;
        const float *conv_dk = dk_in;
        if (with_lkc) {
            // Eq. 5: DK from the unfiltered slice first (Eq. 4 line 2), then F_att (*) LK^c,
            // on which both depth-wise kernels act
            if (gen != nullptr) {
                float *dk = (float *)(w + f.dk_off);
                if ((st = enqueue_dynkernel(x, dt, N, C, H, W, C_a, gen, dk, workspace, f.ws, s)) != ESC_OK) return st;
                conv_gen = nullptr;
                conv_dk = dk;
            }
            PointwiseParams pp{};
            pp.src1 = x;
            pp.src1_img_stride = (size_t)C * plane;
            pp.K1 = C_a;
            pp.w = lk_c;
            pp.w_ld = C_a;
            pp.dst = w + f.pw_off;
            pp.dst_img_stride = (size_t)C_a * plane;
            pp.M = C_a;
            pp.N = N;
            pp.P = (long)plane;
            if (launch_pointwise(pp, bf16, s) != hipSuccess) return ESC_ERR_HIP;
            conv_in = w + f.pw_off;
            conv_c = C_a;
        }
        // F_res = F_pw (*) LK^s + F_pw (*) DK into the workspace; no pass-through copy
        if ((st = enqueue_forward(conv_in, dt, N, conv_c, H, W, C_a, lk, Ks, lk_channel_stride, conv_gen, conv_dk, fres,
                                  C_a, false, workspace, f.ws, s)) != ESC_OK)
            return st;
    }
    // Eq. 4 line 4 (and Eq. 3 line 3): Conv_fuse over F_res and the identity channels of x
    PointwiseParams pp{};
    pp.src1 = fres;
    pp.src1_img_stride = (size_t)C_a * plane;
    pp.K1 = C_a;
    pp.src2 = (const char *)x + (size_t)C_a * plane * es;
    pp.src2_img_stride = (size_t)C * plane;
    pp.K2 = C - C_a;
    pp.w = w_fuse;
    pp.w_ld = C;
    pp.bias = b_fuse;
    pp.res = residual;
    pp.res_img_stride = (size_t)C * plane;
    pp.dst = out;
    pp.dst_img_stride = (size_t)C * plane;
    pp.M = C;
    pp.N = N;
    pp.P = (long)plane;
    return launch_pointwise(pp, bf16, s) == hipSuccess ? ESC_OK : ESC_ERR_HIP;
}

// ---- ConvFFN (Eq. 3 line 3: the feed-forward network in front of the module) ----------

constexpr int kFfnMaxHidden = 960;  // hidden channels (the second layer takes them 224 at a time)

size_t esc_convffn_workspace_bytes(int N, int C_h, int H, int W, esc_dtype dt)
{
    if ((dt != ESC_F32 && dt != ESC_BF16) || N < 1 || C_h < 1 || H < 1 || W < 1) return 0;
    const size_t es = dt == ESC_F32 ? 4 : 2;
    return 2 * round_up((size_t)N * C_h * H * W * es, kWsAlign);  // U and V
}

esc_status esc_convffn_forward(const void *x, esc_dtype dt, int N, int C, int H, int W, int C_h, const float *w1,
                               const float *b1, const float *k_dw, const float *b_dw, const float *w2,
                               const float *b2, void *out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (dt != ESC_F32 && dt != ESC_BF16) return ESC_ERR_DTYPE;
    if (N < 1 || C < 1 || H < 1 || W < 1 || C_h < 1) return ESC_ERR_SHAPE;
    if (x == nullptr || out == nullptr || w1 == nullptr || k_dw == nullptr || w2 == nullptr) return ESC_ERR_NULL;
    if ((size_t)H * (size_t)W >= ((size_t)1 << 31)) return ESC_ERR_UNSUPPORTED;
    if (C > kPointwiseMaxK || C_h > kFfnMaxHidden) return ESC_ERR_UNSUPPORTED;
    const size_t es = dt == ESC_F32 ? 4 : 2;
    const size_t plane = (size_t)H * W;
    // the point-wise kernel addresses an image of a tensor with 32-bit byte offsets
    if ((size_t)C_h * plane * es >= ((size_t)1 << 31) || (size_t)C * plane * es >= ((size_t)1 << 31))
        return ESC_ERR_UNSUPPORTED;
    if (((uintptr_t)x % es) != 0 || ((uintptr_t)out % es) != 0) return ESC_ERR_SHAPE;
    const size_t need = esc_convffn_workspace_bytes(N, C_h, H, W, dt);
    if (workspace == nullptr || ((uintptr_t)workspace % kWsAlign) != 0 || workspace_bytes < need) return ESC_ERR_WORKSPACE;
    const size_t bytes = (size_t)N * C * plane * es;
    if (overlaps(x, bytes, out, bytes) || overlaps(workspace, workspace_bytes, out, bytes) ||
        overlaps(workspace, workspace_bytes, x, bytes))
        return ESC_ERR_ALIAS;
    hipStream_t s = (hipStream_t)stream;
    const bool bf16 = dt == ESC_BF16;
    char *u = (char *)workspace, *v = u + need / 2;
    {
        // up to 64 channels and a hidden layer of up to 128, on an image (or batch) large enough to
        // fill the chip: the whole network in one launch, U and V staying on the chip (the workspace
        // is not touched)
        FfnStreamParams fs{};
        fs.x = x;
        fs.out = out;
        fs.bf16 = bf16 ? 1 : 0;
        fs.w1 = w1, fs.b1 = b1, fs.k = k_dw, fs.bk = b_dw, fs.w2 = w2, fs.b2 = b2;
        fs.N = N, fs.C = C, fs.H = H, fs.W = W, fs.Ch = C_h;
        const hipError_t e = launch_ffn_stream(fs, s);
        if (e == hipSuccess) return ESC_OK;
        if (e != hipErrorNotSupported) return ESC_ERR_HIP;
    }
    // U = gelu(W1 . x + b1)
    PointwiseParams p1{};
    p1.src1 = x;
    p1.src1_img_stride = (size_t)C * plane;
    p1.K1 = C;
    p1.w = w1;
    p1.w_ld = C;
    p1.bias = b1;
    p1.dst = u;
    p1.dst_img_stride = (size_t)C_h * plane;
    p1.M = C_h;
    p1.N = N;
    p1.P = (long)plane;
    p1.gelu = 1;
    if (launch_pointwise(p1, bf16, s) != hipSuccess) return ESC_ERR_HIP;
    // V = U + gelu(K (*) U + bk)
    FfnBranchParams fb{};
    fb.u = u;
    fb.v = v;
    fb.k = k_dw;
    fb.bk = b_dw;
    fb.Ch = C_h;
    fb.H = H;
    fb.W = W;
    fb.planes = (long)N * C_h;
    if (launch_ffn_branch(fb, bf16, s) != hipSuccess) return ESC_ERR_HIP;
    // out = W2 . V + b2; a hidden layer wider than the point-wise kernel's staging holds is multiplied in
    // chunks of its channels, each launch adding to what the launches before it left in out (out as the
    // residual, in place: every element is read and written by the same wavefront)
    constexpr int kChunk = 224;
    for (int k0 = 0; k0 < C_h; k0 += kChunk) {
        PointwiseParams p2{};
        p2.src1 = v + (size_t)k0 * plane * es;
        p2.src1_img_stride = (size_t)C_h * plane;
        p2.K1 = C_h - k0 < kChunk ? C_h - k0 : kChunk;
        p2.w = w2 + k0;
        p2.w_ld = C_h;
        p2.bias = k0 == 0 ? b2 : nullptr;
        p2.res = k0 == 0 ? nullptr : out;
        p2.res_img_stride = (size_t)C * plane;
        p2.dst = out;
        p2.dst_img_stride = (size_t)C * plane;
        p2.M = C;
        p2.N = N;
        p2.P = (long)plane;
        if (launch_pointwise(p2, bf16, s) != hipSuccess) return ESC_ERR_HIP;
    }
    return ESC_OK;
}

// ---- the residual step of Eq. 3 line 3 as one call ---------------------------------

namespace {
struct StepLayout {
    size_t fused, mid_off, ffn_off, total;
};
bool step_layout(int N, int C, int H, int W, int Ca, int Ch, esc_dtype dt, bool with_lkc, StepLayout *l)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || Ch < 1) return false;
    l->fused = esc_fused_workspace_bytes(N, Ca, H, W, dt, with_lkc ? 1 : 0);
    const size_t ffn = esc_convffn_workspace_bytes(N, Ch, H, W, dt);
    if (l->fused == 0 || ffn == 0) return false;
    const size_t es = dt == ESC_F32 ? 4 : 2;
    l->mid_off = round_up(l->fused, kWsAlign);
    l->ffn_off = l->mid_off + round_up((size_t)N * C * H * W * es, kWsAlign);
    l->total = l->ffn_off + ffn;
    return true;
}
}  // namespace

size_t esc_residual_step_workspace_bytes(int N, int C, int H, int W, int C_a, int C_h, esc_dtype dt, int with_lk_c)
{
    StepLayout l;
    if ((dt != ESC_F32 && dt != ESC_BF16) || C_a < 0 || C_a > C) return 0;
    if (!step_layout(N, C, H, W, C_a, C_h, dt, with_lk_c != 0, &l)) return 0;
    return l.total;
}

esc_status esc_residual_step_forward(const void *f_in, esc_dtype dt, int N, int C, int H, int W, int C_h,
                                     const float *w1, const float *b1, const float *k_dw, const float *b_dw,
                                     const float *w2, const float *b2, int C_a, const float *lk_c, const float *lk,
                                     int Ks, long lk_channel_stride, const esc_gen_params *gen, const float *w_fuse,
                                     const float *b_fuse, void *f_out, void *workspace, size_t workspace_bytes,
                                     void *stream)
{
    esc_status st = check_common(f_in, dt, N, C, H, W, C_a);
    if (st != ESC_OK) return st;
    if (C_h < 1) return ESC_ERR_SHAPE;
    if (f_out == nullptr) return ESC_ERR_NULL;
    StepLayout l;
    if (!step_layout(N, C, H, W, C_a, C_h, dt, lk_c != nullptr && C_a > 0, &l)) return ESC_ERR_SHAPE;
    if ((st = check_ws(workspace, workspace_bytes, l.total)) != ESC_OK) return st;
    const size_t es = dt == ESC_F32 ? 4 : 2;
    const size_t bytes = (size_t)N * C * H * W * es;
    if (overlaps(workspace, workspace_bytes, f_out, bytes) || overlaps(workspace, workspace_bytes, f_in, bytes) ||
        overlaps(f_in, bytes, f_out, bytes))
        return ESC_ERR_ALIAS;
    char *w = (char *)workspace;
    void *mid = w + l.mid_off;
    // ConvFFN(F) into the workspace, then F + ConvAttn(that) - every further argument is checked by the two calls,
    // the first of which enqueues nothing before its checks have passed; the second one's arguments that could
    // still fail are checked here first, so that a refused call has enqueued nothing
    if (w_fuse == nullptr || (C_a > 0 && lk == nullptr)) return ESC_ERR_NULL;
    if (Ks < 1 || (Ks % 2) == 0) return Ks < 1 ? ESC_ERR_SHAPE : ESC_ERR_UNSUPPORTED;
    if (Ks > kMaxKs || C > kPointwiseMaxK) return ESC_ERR_UNSUPPORTED;
    if (lk_channel_stride != 0 && lk_channel_stride < (long)Ks * Ks) return ESC_ERR_SHAPE;
    if (gen != nullptr && (st = check_gen(gen, C_a)) != ESC_OK) return st;
    if (((uintptr_t)f_out % es) != 0) return ESC_ERR_SHAPE;
    st = esc_convffn_forward(f_in, dt, N, C, H, W, C_h, w1, b1, k_dw, b_dw, w2, b2, mid, w + l.ffn_off,
                             workspace_bytes - l.ffn_off, stream);
    if (st != ESC_OK) return st;
    return esc_convattn_fused_forward(mid, dt, N, C, H, W, C_a, lk_c, lk, Ks, lk_channel_stride, gen, nullptr, w_fuse,
                                      b_fuse, f_in, f_out, workspace, l.fused, stream);
}

size_t esc_dense_workspace_bytes(int N, int C_a, int H, int W, int Ks)
{
    DenseLayout d;
    if (!dense_layout(N, C_a, H, W, Ks, &d)) return 0;
    return d.total;
}

esc_status esc_convattn_dense_forward(const void *x, esc_dtype dt, int N, int C, int H, int W, int C_a,
                                      const float *lk_dense, int Ks, const esc_gen_params *gen, const float *dk_in,
                                      void *out, void *workspace, size_t workspace_bytes, void *stream)
{
    esc_status st = check_common(x, dt, N, C, H, W, C_a);
    if (st != ESC_OK) return st;
    if (out == nullptr) return ESC_ERR_NULL;
    if (Ks < 1 || (Ks % 2) == 0) return Ks < 1 ? ESC_ERR_SHAPE : ESC_ERR_UNSUPPORTED;
    if (Ks > kDenseMaxKs || C_a > kDenseMaxCa) return ESC_ERR_UNSUPPORTED;
    if (C_a > 0 && lk_dense == nullptr) return ESC_ERR_NULL;
    if (gen != nullptr && (st = check_gen(gen, C_a)) != ESC_OK) return st;
    const size_t es = dt == ESC_F32 ? 4 : 2;
    if (((uintptr_t)out % es) != 0) return ESC_ERR_SHAPE;
    const size_t bytes = (size_t)N * C * H * W * es;
    if (overlaps(x, bytes, out, bytes)) return ESC_ERR_ALIAS;
    DenseLayout d;
    if (!dense_layout(N, C_a, H, W, Ks, &d)) return ESC_ERR_SHAPE;
    if ((st = check_ws(workspace, workspace_bytes, d.total)) != ESC_OK) return st;
    if (overlaps(workspace, workspace_bytes, out, bytes) || overlaps(workspace, workspace_bytes, x, bytes))
        return ESC_ERR_ALIAS;
    if (C_a > 0) {
        if (overlaps(lk_dense, (size_t)C_a * C_a * Ks * Ks * sizeof(float), out, bytes)) return ESC_ERR_ALIAS;
        if (gen == nullptr && dk_in != nullptr && overlaps(dk_in, (size_t)N * C_a * 9 * sizeof(float), out, bytes))
            return ESC_ERR_ALIAS;
    }
    hipStream_t s = (hipStream_t)stream;
    if (C_a == 0)  // nothing but the pass-through copy: the plain forward does that
        return enqueue_forward(x, dt, N, C, H, W, 0, nullptr, Ks, 0, nullptr, nullptr, out, C, true, workspace, d.ws, s);
    char *w = (char *)workspace;
    const float *dk = dk_in;
    float *wt = (float *)(w + d.wt_off);
    bool table_built = false;
    if (gen != nullptr) {  // Eq. 4 line 2: one launch of the variant without conv items
        float *dk_ws = (float *)(w + d.dk_off);
        // (the matrix path's weight table is built by the same launch, beside the pooling)
        table_built = dense_on_bf16_mfma(C_a, Ks, dt == ESC_BF16);
        if ((st = enqueue_dynkernel(x, dt, N, C, H, W, C_a, gen, dk_ws, workspace, d.ws, s, table_built ? lk_dense : nullptr, Ks,
                                    (uint32_t *)wt)) != ESC_OK)
            return st;
        dk = dk_ws;
    }
    if (!table_built && launch_dense_weights(lk_dense, C_a, Ks, dt == ESC_BF16, wt, s) != hipSuccess) return ESC_ERR_HIP;
    DenseParams p{};
    p.x = x;
    p.out = out;
    p.wt = wt;
    p.dk = dk;
    p.N = N;
    p.C = C;
    p.Ca = C_a;
    p.H = H;
    p.W = W;
    p.Ks = Ks;
    p.elem_bytes = (int)es;
    if (C_a < C) {
        const size_t plane = (size_t)H * W * es;
        p.img_bytes = plane * C;
        p.idt_off = plane * C_a;
        p.idt_len = plane * (C - C_a);
        p.copy_vec = ((uintptr_t)x % 16 == 0) && ((uintptr_t)out % 16 == 0) && (p.img_bytes % 16 == 0) &&
                     (p.idt_off % 16 == 0);
    }
    return launch_dense(p, dt == ESC_BF16, s) == hipSuccess ? ESC_OK : ESC_ERR_HIP;
}

size_t esc_backward_workspace_bytes(int N, int C_a, int H, int W, int Ks, int hidden)
{
    BackwardLayout b;
    if (!backward_layout(N, C_a, H, W, Ks, hidden, &b)) return 0;
    return b.total;
}

esc_status esc_convattn_backward(const void *x, const void *grad_out, esc_dtype dt, int N, int C, int H, int W, int C_a,
                                 const float *lk, int Ks, long lk_channel_stride, const esc_gen_params *gen,
                                 const float *dk_in, void *grad_x, float *grad_lk, const esc_gen_grads *grad_gen,
                                 float *grad_dk, int accumulate, void *workspace, size_t workspace_bytes, void *stream)
{
    esc_status st = check_common(x, dt, N, C, H, W, C_a);
    if (st != ESC_OK) return st;
    if (grad_out == nullptr || grad_x == nullptr) return ESC_ERR_NULL;
    if (Ks < 1 || (Ks % 2) == 0) return Ks < 1 ? ESC_ERR_SHAPE : ESC_ERR_UNSUPPORTED;
    if (Ks > kMaxKs) return ESC_ERR_UNSUPPORTED;
    if (C_a > 0 && lk == nullptr) return ESC_ERR_NULL;
    if (lk_channel_stride != 0 && lk_channel_stride < (long)Ks * Ks) return ESC_ERR_SHAPE;
    if (gen != nullptr && (st = check_gen(gen, C_a)) != ESC_OK) return st;
    const size_t es = dt == ESC_F32 ? 4 : 2;
    if (((uintptr_t)grad_out % es) != 0 || ((uintptr_t)grad_x % es) != 0) return ESC_ERR_SHAPE;
    const size_t bytes = (size_t)N * C * H * W * es;
    if (overlaps(x, bytes, grad_x, bytes) || overlaps(grad_out, bytes, grad_x, bytes)) return ESC_ERR_ALIAS;
    const int hidden = gen != nullptr ? gen->hidden : 0;
    BackwardLayout b;
    if (!backward_layout(N, C_a, H, W, Ks, hidden, &b)) return ESC_ERR_SHAPE;
    if ((st = check_ws(workspace, workspace_bytes, b.total)) != ESC_OK) return st;
    if (overlaps(workspace, workspace_bytes, grad_x, bytes) || overlaps(workspace, workspace_bytes, x, bytes) ||
        overlaps(workspace, workspace_bytes, grad_out, bytes))
        return ESC_ERR_ALIAS;
    hipStream_t s = (hipStream_t)stream;
    const bool bf16 = dt == ESC_BF16;
    char *w = (char *)workspace;
    if (C_a == 0)  // no attention channels: the input gradient is the upstream one
        return enqueue_forward(grad_out, dt, N, C, H, W, 0, nullptr, Ks, 0, nullptr, nullptr, grad_x, C, true, workspace,
                               b.ws, s);
    BackwardParams p{};
    p.x = x;
    p.go = grad_out;
    p.N = N;
    p.C = C;
    p.Ca = C_a;
    p.H = H;
    p.W = W;
    p.Ks = Ks;
    p.lk = lk;
    p.lk_cstride = lk_channel_stride;
    p.has_gen = gen != nullptr;
    if (gen != nullptr) {
        p.hidden = gen->hidden;
        p.w_down = gen->w_down;
        p.b_down = gen->b_down;
        p.w_up = gen->w_up;
        p.b_up = gen->b_up;
    } else {
        p.dk_in = dk_in;
    }
    p.partial = (float *)(w + b.partial_off);
    p.ddk = (float *)(w + b.ddk_off);
    p.g = (float *)(w + b.g_off);
    p.t = (float *)(w + b.t_off);
    p.du = (float *)(w + b.du_off);
    p.dgc = (float *)(w + b.dgc_off);
    p.dkf = (float *)(w + b.dkf_off);
    p.lkf = (float *)(w + b.lkf_off);
    p.grad_lk = grad_lk;
    p.grad_dk = grad_dk;
    if (grad_gen != nullptr && gen != nullptr) {
        p.grad_w_down = grad_gen->w_down;
        p.grad_b_down = grad_gen->b_down;
        p.grad_w_up = grad_gen->w_up;
        p.grad_b_up = grad_gen->b_up;
    }
    p.accumulate = accumulate != 0;
    // 1. S = correlation of grad_out with x, per tile (and the tiles' sums of x for the GAP)
    if (launch_backward_sums(p, bf16, s) != hipSuccess) return ESC_ERR_HIP;
    // 2. per image: dL/dDK and the GAP means, the estimator forwards (DK) and backwards; the flipped kernels
    if (launch_backward_estimator(p, s) != hipSuccess) return ESC_ERR_HIP;
    // 3. the sums over the batch: grad_lk and the estimator's parameter gradients
    if (launch_backward_batch_sums(p, s) != hipSuccess) return ESC_ERR_HIP;
    // 4. the input gradient's convolution is the forward on grad_out with the flipped kernels
    //    (identity channels: grad_x = grad_out, the forward's pass-through copy); the GAP's
    //    share, dL/dg / (H W) on every pixel of the attention planes, is added at its stores
    return enqueue_forward(grad_out, dt, N, C, H, W, C_a, p.lkf, Ks, lk_channel_stride != 0 ? (long)Ks * Ks : 0, nullptr,
                           p.dkf, grad_x, C, true, workspace, b.ws, s, p.has_gen ? p.dgc : nullptr);
}

const char *esc_status_string(esc_status s)
{
    switch (s) {
    case ESC_OK: return "ok";
    case ESC_ERR_NULL: return "a required pointer is NULL";
    case ESC_ERR_SHAPE: return "a size or stride is out of its domain";
    case ESC_ERR_DTYPE: return "unknown storage type";
    case ESC_ERR_UNSUPPORTED: return "outside the library's limits (Ks odd <= 31, C_a <= 256, hidden <= 256; fused call: C <= 240; dense call: C_a <= 64, Ks <= 17)";
    case ESC_ERR_WORKSPACE: return "workspace missing, misaligned or too small (esc_convattn_forward_noalloc: shape beyond the built-in scratch)";
    case ESC_ERR_ALIAS: return "out overlaps x, the workspace, lk or dk";
    case ESC_ERR_HIP: return "the HIP runtime refused a launch";
    case ESC_STATUS_INT_RANGE: break;
    }
    return "unknown status";
}

}  // extern "C"

/*
 * esc_convattn.h - C ABI of the MI355X (gfx950) ConvAttn forward library.
 *
 * The operation is the Convolutional Attention Module of the ESC paper
 * (Sec. 3, Eq. 4) with the depth-wise large kernel LK^s of the paragraph that
 * introduces Eq. 5, stopped before the 1x1 fuse convolution:
 *
 *   F_att, F_idt = Split(x)                 first C_a channels / the rest   (Eq. 4 line 1)
 *   DK           = Estimator(GAP(F_att))    one 3x3 kernel per image+channel (Eq. 4 line 2)
 *   F_res        = F_att (*) DK + F_att (*) LK                               (Eq. 4 line 3)
 *   out          = Concat(F_res, F_idt)                                      (Eq. 4 line 4)
 *
 * (*) is depth-wise cross-correlation, zero padding (K-1)/2, stride 1, so the
 * output keeps H x W.  Accumulation is fp32; F_res is rounded once, at the
 * store, to the storage type.  F_idt is copied bit for bit.
 *
 * Conventions shared by every entry point
 *   - All data pointers are DEVICE pointers, caller-owned, never freed, copied
 *     or retained by the library.  `stream` is a hipStream_t passed as void*
 *     (NULL = the default stream).  Calls only enqueue work on `stream` and
 *     return; they never synchronise and never allocate.
 *   - x and out are contiguous [N, C, H, W] in the storage type `dt`; out must
 *     not overlap x, the workspace, lk, dk_in or dk_out (ESC_ERR_ALIAS for the
 *     ranges the library can see).  lk, the estimator weights, dk and the
 *     workspace are fp32 in both storage modes.  With bf16 storage and Ks <= 17
 *     the large-kernel weights are rounded to bf16 on the device before use
 *     (products are exact, accumulation stays fp32) and the taps run on the
 *     matrix cores, 16 neighbouring outputs of a row from 32 input columns at a
 *     time, most of them times a zero: a pixel of the attention slice that is
 *     not finite then turns into NaN, in the rows its kernel window reaches,
 *     every such run of 16 outputs (columns 16 b ... 16 b + 15) whose 32 input
 *     columns hold it, and nothing else.  fp32 storage, and bf16 storage with
 *     Ks >= 19, give NaN/Inf exactly where the definition does.
 *   - All arguments are validated on the host before the first launch; a call
 *     that returns an error has enqueued nothing.
 *   - Every compute call needs a workspace (work queue and the mailboxes blocks
 *     use to hand over the GAP sums and DK).  It must have been prepared once with
 *     esc_workspace_init on a stream ordered before its first use; calls leave it
 *     ready for the next call, whatever its shape, so it carries state from call
 *     to call and must not be cleared or reused for anything else in between.
 *     esc_workspace_bytes gives the size for a shape; it never shrinks when N,
 *     C_a, H or W grow (each taken by itself - not H*W), so a workspace sized
 *     for the largest N, C_a, H and W fits every smaller shape.
 *   - The forward is one persistent kernel whose blocks wait for one another
 *     (bounded, about a second).  Its grid is sized, per device and kernel
 *     variant, from the runtime's occupancy answer so that all of its blocks are
 *     resident at once on an otherwise idle device (ESC_ERR_UNSUPPORTED if the
 *     device cannot hold one block).  Calls of this library on DIFFERENT streams
 *     must be serialised by the caller (two half-resident grids could wait for
 *     each other), and other work that keeps running on the same device at the
 *     same time can hold blocks back and stretch the waits.  Should a wait ever
 *     expire, the values that never came are taken as NaN - the affected outputs
 *     are NaN, never silently wrong numbers - and the workspace's error word is
 *     raised; esc_workspace_errors reads it.
 *   - Limits: 0 <= C_a <= min(C, 256); estimator hidden width <= 256; Ks odd,
 *     1 <= Ks <= 31; H*W < 2^31; N, C, H, W >= 1.  No lower bound on H or W
 *     relative to Ks.
 */
#ifndef ESC_CONVATTN_H
#define ESC_CONVATTN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ESC_OK = 0,
    ESC_ERR_NULL = 1,        /* a required pointer is NULL                         */
    ESC_ERR_SHAPE = 2,       /* a size is out of its domain (N<1, C_a>C, ...)      */
    ESC_ERR_DTYPE = 3,       /* dt is not a member of esc_dtype                    */
    ESC_ERR_UNSUPPORTED = 4, /* valid for the method, outside the library's limits */
    ESC_ERR_WORKSPACE = 5,   /* workspace missing, misaligned or too small         */
    ESC_ERR_ALIAS = 6,       /* out overlaps x, the workspace, lk, dk_in or dk_out  */
    ESC_ERR_HIP = 7,         /* the HIP runtime refused a launch                   */
    ESC_STATUS_INT_RANGE = 0x7fffffff /* not a status: gives the type the range of int */
} esc_status;

/* storage type of x and out (the last member is not a type: it gives the enum the range of
 * int, so that a bad value is an argument to refuse, not undefined behaviour) */
typedef enum { ESC_F32 = 0, ESC_BF16 = 1, ESC_DTYPE_INT_RANGE = 0x7fffffff } esc_dtype;

/*
 * The kernel estimator of Eq. 4 line 2, applied to g = GAP(F_att) of one image:
 *   hidden == 0 : d = w_up[9*C_a, C_a] g + b_up                 (single linear layer)
 *   hidden  > 0 : d = w_up[9*C_a, hidden] gelu(w_down[hidden, C_a] g + b_down) + b_up
 * gelu is the exact erf form.  Matrices are row-major [out, in], fp32, device
 * memory.  Either bias may be NULL (zero).  DK[c, i, j] = d[c*9 + i*3 + j].
 */
typedef struct esc_gen_params {
    int hidden;
    const float *w_down; /* [hidden, C_a]; ignored when hidden == 0 */
    const float *b_down; /* [hidden] or NULL                        */
    const float *w_up;   /* [9*C_a, hidden ? hidden : C_a]          */
    const float *b_up;   /* [9*C_a] or NULL                         */
} esc_gen_params;

/* Bytes of workspace a call with this shape needs (256-byte aligned base). 0 on bad arguments. */
size_t esc_workspace_bytes(int N, int C_a, int H, int W);

/* Prepare a freshly allocated workspace (enqueues one small fill kernel on `stream`). */
esc_status esc_workspace_init(void *workspace, size_t workspace_bytes, void *stream);

/*
 * Diagnostic, not part of the hot path: copies the workspace's error word to
 * *errors_out (HOST pointer) and SYNCHRONISES `stream` to do so.  0 = no wait has
 * expired in any call since esc_workspace_init.
 */
esc_status esc_workspace_errors(const void *workspace, size_t workspace_bytes, void *stream,
                                unsigned *errors_out);

/*
 * Eq. 4 line 2 alone: GAP over the attention slice, then the estimator.
 *   x       [N,C,H,W] storage type dt (read)      dk_out [N,C_a,3,3] fp32 (written)
 * C_a == 0 is accepted and does nothing.
 */
esc_status esc_dynkernel_gen(const void *x, esc_dtype dt, int N, int C, int H, int W, int C_a,
                             const esc_gen_params *gen, float *dk_out,
                             void *workspace, size_t workspace_bytes, void *stream);

/*
 * Eq. 4 lines 1-4 (without Conv_fuse).
 *   lk     [C_a, Ks, Ks] fp32, channel c at lk + c*lk_channel_stride; a stride of
 *          0 applies one Ks x Ks filter to every channel; otherwise >= Ks*Ks.
 *   gen    estimator weights; when non-NULL, DK is computed from x (dk_in ignored)
 *   dk_in  [N,C_a,3,3] fp32 DK used as given when gen is NULL; both NULL => DK = 0
 *   out    [N,C,H,W] storage type dt (written, every element)
 * With gen != NULL the result equals esc_dynkernel_gen followed by this call
 * with dk_in, bit for bit.
 */
esc_status esc_convattn_forward(const void *x, esc_dtype dt, int N, int C, int H, int W, int C_a,
                                const float *lk, int Ks, long lk_channel_stride,
                                const esc_gen_params *gen, const float *dk_in,
                                void *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The module with its point-wise steps (Eq. 4 lines 1-4 in full; Eq. 5; Eq. 3 line 3):
 *
 *   F_pw  = F_att (*) LK^c                  lk_c [C_a, C_a] row-major [out, in], 1x1, no bias;
 *                                            NULL = F_att itself (Eq. 4 line 3 as it stands)
 *   DK    = Estimator(GAP(F_att))           from the UNFILTERED slice (Eq. 4 line 2)
 *   F_res = F_pw (*) (ZP(DK) + LK^s)        depth-wise, as in esc_convattn_forward (Eq. 5)
 *   out   = Conv_fuse(Concat(F_res, F_idt)) w_fuse [C, C] row-major [out, in], b_fuse [C] or NULL
 *           + residual                      [N,C,H,W] in the storage type, or NULL (Eq. 3 line 3:
 *                                            the tensor the module's result is added to)
 *
 * The concat is never written: Conv_fuse reads F_res from the workspace and the identity
 * channels from x, on the matrix cores: with fp32 storage fp32 products and fp32
 * accumulation; with bf16 storage bf16 matrix instructions on the stored values, each fp32
 * weight applied as the sum of two bf16 terms (w = hi + lo to 16 mantissa bits; products
 * exact, accumulation fp32).  F_res (and F_pw) pass through the workspace in the storage
 * type, so with bf16 storage they are rounded to bf16 on the way, as a network's tensors
 * would be; out is rounded once more at its store.  out must not overlap x, residual or
 * the workspace.  The workspace is larger than esc_convattn_forward's
 * (esc_fused_workspace_bytes; with_lk_c != 0 when lk_c will be given), prepared with the
 * same esc_workspace_init, and serves esc_convattn_forward / esc_dynkernel_gen calls of
 * the same shape as well.  Limits as above, and C <= 240.  Two to four launches on `stream`.
 */
size_t esc_fused_workspace_bytes(int N, int C_a, int H, int W, esc_dtype dt, int with_lk_c);
esc_status esc_convattn_fused_forward(const void *x, esc_dtype dt, int N, int C, int H, int W, int C_a,
                                      const float *lk_c, const float *lk, int Ks, long lk_channel_stride,
                                      const esc_gen_params *gen, const float *dk_in,
                                      const float *w_fuse, const float *b_fuse, const void *residual,
                                      void *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * ConvFFN, the feed-forward network whose output the module takes in the residual step
 * F_{i,j} = F_{i,j-1} + ConvAttn_j(ConvFFN_j(F_{i,j-1}), LK)  (Eq. 3 line 3).  Sec. 3 names it
 * (the convolutional feed-forward network of the work the paper cites, kernel size three)
 * and prints no equation; as that network is described - two point-wise layers with a
 * depth-wise convolution branch between them:
 *
 *   U   = gelu(w1 . x + b1)            w1 [C_h, C] row-major, b1 [C_h] or NULL; the erf form of
 *                                      GELU (not its tanh approximation), erf evaluated to 1.5e-7
 *   V   = U + gelu(k_dw (*) U + b_dw)  k_dw [C_h, 3, 3] depth-wise, cross-correlation, zero
 *                                      padding 1; b_dw [C_h] or NULL
 *   out = w2 . V + b2                  w2 [C, C_h] row-major, b2 [C] or NULL
 *
 *   x, out    [N,C,H,W] in the storage type (device); out must not overlap x or the workspace
 *   C_h       width of the hidden layer (the paper does not print its ratio to C)
 * All weights are device pointers to fp32, read-only.  The point-wise layers run on the
 * matrix cores as in esc_convattn_fused_forward (fp32 storage: fp32 products; bf16 storage:
 * bf16 instructions on the stored values, each fp32 weight as two bf16 terms), the branch
 * in fp32 on the vector units.  With C <= 64, C_h <= 128, an image (or batch) large enough
 * to fill the chip with 30-column strips and a width that fills at least four fifths of its
 * strips, the call takes ONE launch in which U and V
 * never leave the chip (the workspace is not touched; with bf16 storage U stays fp32 and V
 * is rounded to bf16 once, as the second layer's operand); everything else takes three
 * launches, U and V passing through the workspace in the storage type, so that with bf16
 * storage both are rounded to bf16 on the way.  out is rounded once at its store.
 * The workspace (esc_convffn_workspace_bytes, 256-byte aligned) is plain scratch: it needs
 * no esc_workspace_init and its contents are undefined after the call.  Limits: C <= 240,
 * C_h <= 960, C_h*H*W*element size < 2 GiB.  A hidden layer of more than 224 channels is
 * multiplied by w2 224 channels at a time, each launch adding to out (with bf16 storage the
 * partial sums are rounded to bf16 between the launches).  The whole residual step is this call followed by
 * esc_convattn_fused_forward on its output with residual = x.
 */
size_t esc_convffn_workspace_bytes(int N, int C_h, int H, int W, esc_dtype dt);
esc_status esc_convffn_forward(const void *x, esc_dtype dt, int N, int C, int H, int W, int C_h,
                               const float *w1, const float *b1, const float *k_dw, const float *b_dw,
                               const float *w2, const float *b2,
                               void *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The residual step of the ESC block as one call (Eq. 3 line 3):
 *
 *   f_out = f_in + ConvAttn(ConvFFN(f_in), LK)
 *
 * i.e. esc_convffn_forward on f_in (its result stays in the workspace, in the storage type),
 * then esc_convattn_fused_forward on that result with residual = f_in; every argument means
 * what it means in those two calls (the estimator `gen` may be NULL: then DK = 0).  f_out must
 * not overlap f_in or the workspace.  The workspace (esc_residual_step_workspace_bytes;
 * with_lk_c != 0 when lk_c will be given) is prepared once with esc_workspace_init; it begins
 * with the fused call's workspace, so esc_workspace_errors applies to it.  All arguments are
 * checked before anything is enqueued.  Launches: those of the two calls (three to eight).
 */
size_t esc_residual_step_workspace_bytes(int N, int C, int H, int W, int C_a, int C_h, esc_dtype dt, int with_lk_c);
esc_status esc_residual_step_forward(const void *f_in, esc_dtype dt, int N, int C, int H, int W, int C_h,
                                     const float *w1, const float *b1, const float *k_dw, const float *b_dw,
                                     const float *w2, const float *b2,
                                     int C_a, const float *lk_c, const float *lk, int Ks, long lk_channel_stride,
                                     const esc_gen_params *gen, const float *w_fuse, const float *b_fuse,
                                     void *f_out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Eq. 4 lines 1-4 (without Conv_fuse) with the DENSE large kernel of the paper's main
 * variants (Sec. 3: LK in R^{Ks x Ks x C_a x C_a}, shared by the whole model):
 *
 *   F_res[co] = sum_ci F_att[ci] (*) LK[co, ci]  +  F_att[co] (*) DK[co]
 *
 *   lk_dense [C_a, C_a, Ks, Ks] fp32, output channel first; cross-correlation, zero padding.
 * DK stays a separate depth-wise term, as in the paper.  Everything else (gen, dk_in, out,
 * the identity channels, rounding) is as in esc_convattn_forward.  The contraction runs on
 * the matrix cores with fp32 accumulation.  With C_a <= 16 on the bf16 matrix instructions:
 * bf16 storage on the stored values, each fp32 weight applied as the sum of two bf16 terms
 * (w = hi + lo to 16 mantissa bits; products exact); fp32 storage with Ks <= 13 on values and
 * weights each split exactly into three bf16 terms, the six products of terms whose orders
 * add up to at most two accumulated (what is left out lies below 2^-24 of a product: fp32
 * accuracy).  Otherwise fp32 instructions (bf16 storage widened exactly).  Limits:
 * C_a <= 64, Ks odd <= 17.
 * The workspace is esc_dense_workspace_bytes large (the forward's workspace, DK and the
 * rearranged weights), prepared with esc_workspace_init.  Two or three launches on `stream`.
 */
size_t esc_dense_workspace_bytes(int N, int C_a, int H, int W, int Ks);
esc_status esc_convattn_dense_forward(const void *x, esc_dtype dt, int N, int C, int H, int W, int C_a,
                                      const float *lk_dense, int Ks,
                                      const esc_gen_params *gen, const float *dk_in,
                                      void *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Backward of esc_convattn_forward (the paper trains its shared LK end to end, Sec. 3; it
 * prints no gradient formulae - these are the derivatives of Eq. 4 lines 1-4 as defined
 * above).  Given grad_out = dL/dout [N,C,H,W] in the storage type:
 *
 *   grad_x   [N,C,H,W] storage type (written, every element): identity channels = grad_out;
 *            attention channels = grad_out (*) flipped (LK + ZP(DK)) + the GAP path's
 *            dL/dg / (H W)
 *   grad_lk  fp32, laid out like lk (same channel stride; ONE Ks x Ks filter, summed over
 *            the channels, when lk_channel_stride == 0), summed over the batch; or NULL
 *   grad_gen gradients of the estimator's weights (each member fp32, shaped like the
 *            weight, or NULL); ignored when gen is NULL
 *   grad_dk  [N,C_a,3,3] fp32, dL/dDK (what a caller who supplied dk_in needs); or NULL
 *   accumulate != 0: the parameter gradients (grad_lk, grad_gen) are ADDED to the buffers'
 *            contents - the way a kernel shared by many modules collects its gradient
 * x, lk, gen and dk_in are the forward's inputs.  fp32 accumulation throughout; every sum
 * has a fixed order.  grad_lk's correlation of grad_out with x runs, for Ks <= 15, on the
 * bf16 matrix instructions with exact products: bf16 values as they are, fp32 values each
 * split into three bf16 terms (exactly, but for values below 2^-102), all nine products of
 * terms accumulated.  The workspace is esc_backward_workspace_bytes large, prepared with
 * esc_workspace_init.  Four launches on `stream`.
 */
typedef struct esc_gen_grads {
    float *w_down; /* [hidden, C_a] or NULL */
    float *b_down; /* [hidden] or NULL      */
    float *w_up;   /* [9*C_a, hidden ? hidden : C_a] or NULL */
    float *b_up;   /* [9*C_a] or NULL       */
} esc_gen_grads;
size_t esc_backward_workspace_bytes(int N, int C_a, int H, int W, int Ks, int hidden);
esc_status esc_convattn_backward(const void *x, const void *grad_out, esc_dtype dt, int N, int C, int H, int W,
                                 int C_a, const float *lk, int Ks, long lk_channel_stride,
                                 const esc_gen_params *gen, const float *dk_in,
                                 void *grad_x, float *grad_lk, const esc_gen_grads *grad_gen, float *grad_dk,
                                 int accumulate, void *workspace, size_t workspace_bytes, void *stream);

/*
 * For callers that cannot allocate or prepare device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): esc_convattn_forward
 * without the workspace arguments.  The mailboxes and counters live in a scratch array
 * inside the library, ESC_NOALLOC_SCRATCH_BYTES per device, which needs no
 * esc_workspace_init.  The call allocates nothing and computes exactly what
 * esc_convattn_forward computes, bit for bit.  Shapes whose esc_workspace_bytes exceeds
 * ESC_NOALLOC_SCRATCH_BYTES are refused with ESC_ERR_WORKSPACE (all arguments are checked
 * as in esc_convattn_forward, before anything is enqueued).  Every call on a device uses
 * that device's one array, which carries state from call to call: calls that overlap on
 * one device (different streams, different threads) race; order them.
 */
#define ESC_NOALLOC_SCRATCH_BYTES (1u << 20)
esc_status esc_convattn_forward_noalloc(const void *x, esc_dtype dt, int N, int C, int H, int W, int C_a,
                                        const float *lk, int Ks, long lk_channel_stride,
                                        const esc_gen_params *gen, const float *dk_in,
                                        void *out, void *stream);

/* Static, NUL-terminated description of a status code. */
const char *esc_status_string(esc_status s);

#ifdef __cplusplus
}
#endif
#endif /* ESC_CONVATTN_H */

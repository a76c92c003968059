/*
 * omniconv -- batched-lowering convolution for one MI355X (gfx950), C ABI.
 *
 * The library computes a convolution layer the way the paper's single-node engine does
 * (Omnivore, arXiv 1606.04487, Sec. III-B "Batching and Data Parallelism" and App. C
 * "Convolution by Lowering and GEMM"): the WHOLE mini-batch is lowered into one matrix
 * D-hat and each pass of the layer is ONE dense matrix product on the matrix cores.
 *
 * Conventions for every entry point
 *   - Pointers named X, W, Y, dX, dY, dW, bias, workspace, ... are DEVICE pointers owned by the
 *     caller (for example a torch tensor's data_ptr()).  The library never allocates, frees or
 *     keeps them.  Descriptors, shape outputs and the pointer tables of omni_sgd_momentum_step
 *     are HOST memory.
 *   - Tensors are dense and contiguous: X [N][C][H][W], W [F][C][kh][kw], Y [N][F][Ho][Wo].
 *     `dtype` is the storage type of X, W, Y, dY, dX and of D-hat; products are accumulated in
 *     fp32 on the matrix cores and rounded to nearest-even once on store.  bias, dW, dbias and
 *     the optimizer state are always fp32.
 *   - Outputs are overwritten, never accumulated into.  Results are deterministic: no floating
 *     point atomics are used, so equal inputs give bit-identical outputs.
 *   - Calls only enqueue work on `hip_stream` (a hipStream_t passed as void*, NULL = the null
 *     stream) and return; nothing synchronises with the device.
 *   - Device pointers must be 16-byte aligned (OMNI_MISALIGNED otherwise).
 *   - Return value: OMNI_OK (0) or a negative omni_status.  Argument checks are done on the
 *     host before anything is launched; a failed call launches nothing.
 */
#ifndef OMNICONV_H
#define OMNICONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    OMNI_OK = 0,
    OMNI_INVALID_ARGUMENT = -1,    /* null required pointer, non-positive extent, empty output  */
    OMNI_UNSUPPORTED = -2,         /* unknown dtype or flag, extents beyond 32-bit indexing     */
    OMNI_WORKSPACE_TOO_SMALL = -3, /* workspace_bytes below omni_conv_workspace_bytes()         */
    OMNI_MISALIGNED = -4,          /* a device pointer is not 16-byte aligned                   */
    OMNI_HIP_ERROR = -5            /* the HIP runtime refused a launch                           */
} omni_status;

typedef enum { OMNI_F32 = 0, OMNI_BF16 = 1 } omni_dtype;

typedef enum {
    OMNI_PASS_FORWARD = 0,
    OMNI_PASS_BACKWARD_DATA = 1,
    OMNI_PASS_BACKWARD_WEIGHTS = 2
} omni_pass;

/* omni_conv_desc.flags */
#define OMNI_FLAG_RELU 1u        /* forward: store max(0, .) (ReLU fused into the GEMM epilogue) */
#define OMNI_FLAG_DHAT_CACHED 2u /* backward_weights: the workspace still holds D-hat written by
                                    omni_conv_forward for the same descriptor and the same X, so
                                    the lowering pass is skipped (the paper's b_p = b: with 288 GB
                                    of HBM every layer's D-hat can stay resident)                */
#define OMNI_FLAG_FUSED 4u       /* every pass: where omni_conv_fused_supported() says so, compute the
                                    same result without D-hat / dD-hat in memory (App. C names fusing
                                    lowering and GEMM as the way past the replication cost of the
                                    lowering phase).  forward / backward_data: lowering, resp. col2im, is
                                    folded into the matrix product.  backward_weights (unless
                                    OMNI_FLAG_DHAT_CACHED is also set): the product reads the entries of
                                    D-hat straight from X.  The workspace then holds no D-hat afterwards.
                                    Elsewhere the flag is ignored and the explicit path runs.            */
#define OMNI_FLAG_SPLIT_K 8u     /* forward / backward_data, explicit path: when the result alone has too
                                    few tiles to occupy the chip (few images per product: a small b_p of
                                    Sec. III-B, or the fully connected layers run as whole-image
                                    convolutions), split the product's reduction over the compute units:
                                    fp32 partial results in the workspace, added in split order by a second
                                    kernel that also applies bias / ReLU and stores.  Deterministic; differs
                                    from the unsplit product by the fp32 rounding of another summation order.
                                    Needs more workspace (omni_conv_workspace_bytes accounts for it).     */

/*
 * A convolution layer (Sec. III-A, Eq. (conv_full); App. C adds stride and zero padding):
 *   Y[n,f,oy,ox] = bias[f] + sum_{c,ky,kx} X[n,c,oy*stride_h-pad_h+ky,ox*stride_w-pad_w+kx] * W[f,c,ky,kx]
 * with X read as zero outside the image, no kernel flip, Ho = (H+2*pad_h-kh)/stride_h + 1
 * (integer division; windows that do not fit are dropped), Wo likewise.  Groups and dilation
 * are fixed at 1 (the paper removes grouping from its networks).
 */
typedef struct {
    int32_t N, C, H, W;
    int32_t F, kh, kw;
    int32_t stride_h, stride_w, pad_h, pad_w;
    int32_t dtype;   /* omni_dtype */
    uint32_t flags;  /* OMNI_FLAG_* */
} omni_conv_desc;

/* Host only.  Writes Ho, Wo.  OMNI_INVALID_ARGUMENT if any extent is non-positive, padding is
 * negative or the window does not fit the padded image. */
int omni_conv_output_dims(const omni_conv_desc *desc, int32_t *Ho, int32_t *Wo);

/* Host only.  Leading dimension (in elements) of D-hat inside the workspace: N*Ho*Wo rounded up
 * to a multiple of 64.  omni_lower / omni_col2im take the leading dimension as an argument. */
int omni_conv_dhat_ld(const omni_conv_desc *desc, int64_t *ld);

/* Host only.  Bytes of scratch the given pass (omni_pass) needs.  The forward and
 * backward-weights workspaces both begin with D-hat ([C*kh*kw][ld], desc->dtype), which is what
 * makes OMNI_FLAG_DHAT_CACHED possible when the same buffer is passed to both. */
int omni_conv_workspace_bytes(const omni_conv_desc *desc, int pass, size_t *bytes);

/* Host only.  1 if the pass (omni_pass) of this layer runs fused under OMNI_FLAG_FUSED, 0 if it
 * falls back to the explicit path, negative status for a bad descriptor.  Fused forward and
 * backward_data: bf16, stride 1, reduced channels a multiple of 32, and the pixels needed by 256
 * consecutive output positions fit the kernel's LDS patch (and the layer is not one that backward_data
 * handles as a single dense product, see there).  Fused backward_weights: bf16, stride 1, a result that
 * fills 256 x 256 or 384 x 128 tiles.  Layers with horizontal stride 4, no padding and at most 96 filters
 * (bf16; CaffeNet's conv1) run fused too: forward when C * kh * ceil(kw / 4) <= 100 and the input rows of 512
 * output positions fit the kernel's LDS patch; backward_weights when 4 * C * kh * ceil(kw / 4) < 512 and
 * Wo >= 8 (the input is split into its four column phases in the workspace and the product reads those and
 * dY as they are; the bias gradient comes out of the same product).  backward_data of any strided, unpadded
 * bf16 layer with F a multiple of 32 runs as one fused stride-1 convolution over dY with C * stride_h *
 * stride_w output channels (one per input channel and pixel phase) followed by the interleaving of the phase
 * images into dX, provided that convolution meets the stride-1 conditions above.
 * The workspace size of a pass does not depend on OMNI_FLAG_FUSED. */
int omni_conv_fused_supported(const omni_conv_desc *desc, int pass);

/*
 * Forward pass (Sec. III-B: lower all N images, then a single GEMM; App. C: lifting is pure
 * addressing and costs no copy).  Steps: batched lowering of X into the workspace, reshaping of
 * W into a padded K-hat (W itself where K needs no padding), one MFMA GEMM
 * Y-hat[F x M] = K-hat[F x K] * D-hat[K x M] whose epilogue adds bias (nullable, fp32[F]), applies ReLU if
 * OMNI_FLAG_RELU and stores straight into Y [N][F][Ho][Wo].  With OMNI_FLAG_SPLIT_K a product with few
 * columns splits its reduction (see the flag).
 */
int omni_conv_forward(const omni_conv_desc *desc, const void *X, const void *W, const float *bias,
                      void *Y, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * omni_conv_forward for callers that cannot allocate device memory and have no workspace to hand over: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (minus the
 * workspace), same kernels and bit-identical results; the scratch is an array of OMNI_STATIC_SCRATCH_BYTES that
 * is part of the library's device code, so every GPU the library runs on holds one copy of it from load time
 * until the process ends.  The call itself allocates nothing and frees nothing (keep omni_profile_enable off:
 * profiling creates events).  omni_conv_static_scratch_need (host only) tells how many bytes of scratch the path
 * this descriptor takes would use: the repacked weights of a fused pass, or D-hat + K-hat (+ split partials) of
 * the explicit path.  A layer that needs more than OMNI_STATIC_SCRATCH_BYTES is refused with
 * OMNI_WORKSPACE_TOO_SMALL before anything is launched; use omni_conv_forward with a workspace for it.
 * Every call on a GPU uses that GPU's one array: calls that overlap on the same GPU (two streams, two threads)
 * race on it and must be ordered by the caller.  Nothing in the array has to be zero beforehand: each call
 * writes every byte it later reads, so the previous call's contents never matter.
 */
#define OMNI_STATIC_SCRATCH_BYTES (32u << 20)
int omni_conv_static_scratch_need(const omni_conv_desc *desc, size_t *bytes);
int omni_conv_forward_static(const omni_conv_desc *desc, const void *X, const void *W, const float *bias,
                             void *Y, void *hip_stream);

/*
 * Forward pass with partial batching (Sec. III-B, "Batching and Data Parallelism": b_p of the b images are
 * lowered and multiplied at a time; App. C, Fig. (b), (c): the lowered data grows linearly with b_p and one
 * large product beats many small ones).  Runs omni_conv_forward's explicit path on consecutive groups of
 * b_p images (the last group may be smaller) through ONE workspace sized for b_p images:
 * workspace_bytes >= omni_conv_workspace_bytes of the same descriptor with N = b_p (and, with
 * OMNI_FLAG_SPLIT_K, also of the one with N = the smaller last group, N mod b_p).  Without OMNI_FLAG_SPLIT_K
 * every output element is the same sum in the same order for every b_p, so Y is bit-identical to
 * omni_conv_forward's; with it the split, hence the rounding, depends on the group's size.
 * 1 <= b_p <= N; for b_p < N a group of b_p images of X and of Y must be a multiple of 16 bytes (OMNI_MISALIGNED
 * otherwise).  OMNI_FLAG_FUSED is ignored: the knob is about D-hat's footprint.
 */
int omni_conv_forward_partial(const omni_conv_desc *desc, int32_t b_p, const void *X, const void *W,
                              const float *bias, void *Y, void *workspace, size_t workspace_bytes,
                              void *hip_stream);

/*
 * Data gradient (Sec. II-B: BW maps the gradient w.r.t. the layer's output to the gradient
 * w.r.t. its input).  Steps: dY is packed into the matrix dY-hat [F][ld]; one MFMA GEMM
 * dD-hat[K x M] = K-hat^T[K x F] * dY-hat[F x M]; col2im sums the entries of dD-hat that were copies
 * of the same input pixel into dX [N][C][H][W] (gather form, fixed summation order).
 * A layer whose window is the whole unpadded image (Ho = Wo = 1: a fully connected layer, Sec. II-C) with F
 * and K multiples of 8 takes one product dX [N][K] = dY [N][F] * W [F][K] on the tensors as they are instead.
 * OMNI_FLAG_SPLIT_K applies to either form.
 */
int omni_conv_backward_data(const omni_conv_desc *desc, const void *dY, const void *W, void *dX,
                            void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Model gradient, summed over the images of the batch with no 1/N (Sec. II-B).  Steps: lowering of X (skipped with OMNI_FLAG_DHAT_CACHED), packing of dY, one MFMA
 * GEMM dK-hat[F x K] = dY-hat[F x M] * D-hat^T[M x K] split along M over the chip with a second,
 * ordered reduction stage.  dW is fp32 [F][C][kh][kw]; dbias (nullable) is fp32 [F] and receives
 * the plain sum of dY over images and pixels.
 */
int omni_conv_backward_weights(const omni_conv_desc *desc, const void *X, const void *dY, float *dW,
                               float *dbias, void *workspace, size_t workspace_bytes,
                               void *hip_stream);

/*
 * Repacked weights as an object of the caller's (App. C: the model, unlike the data, needs no replication -- it
 * only changes once per step).  With OMNI_FLAG_FUSED the forward pass and the data gradient read the weights in
 * kernel-specific orders, which omni_conv_forward / omni_conv_backward_data write into their workspace on every
 * call.  A caller whose weights change once per training step can instead keep those copies itself:
 *   omni_conv_packed_weights_bytes: bytes of the copy that `pass` (OMNI_PASS_FORWARD or OMNI_PASS_BACKWARD_DATA) of
 *       this layer reads; 0 when that pass does not read repacked weights (then the *_packed calls below return
 *       OMNI_UNSUPPORTED for it and the plain entry points are the ones to call).  Host only.
 *   omni_conv_pack_weights: ONE launch that writes the copies of n layer-and-pass pairs (n <= 16): descs is a host
 *       array of n descriptors, passes of n pass ids, W and packed host arrays of n device pointers (W[i] the
 *       layer's bf16 weights [F][C][kh][kw], packed[i] the caller's buffer of omni_conv_packed_weights_bytes).
 *       An entry whose pass reads no repacked weights is OMNI_UNSUPPORTED (nothing is launched).
 *   omni_conv_forward_packed / omni_conv_backward_data_packed: omni_conv_forward / omni_conv_backward_data with
 *       `packed` (as written by omni_conv_pack_weights for the same descriptor and pass) in place of W; results are
 *       bit-identical to the plain entry points'.  Workspace as for the plain entry points.
 * All pointers 16-byte aligned; the copies stay valid until W changes.
 */
int omni_conv_packed_weights_bytes(const omni_conv_desc *desc, int pass, size_t *bytes);
int omni_conv_pack_weights(int32_t n, const omni_conv_desc *descs, const int32_t *passes, const void *const *W,
                           void *const *packed, void *hip_stream);
int omni_conv_forward_packed(const omni_conv_desc *desc, const void *X, const void *packed, const float *bias,
                             void *Y, void *workspace, size_t workspace_bytes, void *hip_stream);
int omni_conv_backward_data_packed(const omni_conv_desc *desc, const void *dY, const void *packed, void *dX,
                                   void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Momentum SGD over a list of parameter tensors in one launch sequence
 * (Sec. II-B, Eq. (update2) then Eq. (update1)):
 *     V <- momentum * V - lr * (G + weight_decay * W);    W <- W + V
 * W, V, G and W_shadow are HOST arrays of n_tensors DEVICE pointers; counts (host) holds each
 * tensor's element count.  W and V are updated in place, G is read.  W_shadow is nullable, and
 * so is each of its entries; where given, the updated W is also stored there as bf16 (the copy
 * the bf16 forward pass reads).  n_tensors == 0 is a no-op; counts[i] == 0 skips tensor i.
 */
int omni_sgd_momentum_step(int32_t n_tensors, float *const *W, float *const *V,
                           const float *const *G, const int64_t *counts, void *const *W_shadow,
                           float lr, float momentum, float weight_decay, void *hip_stream);

/*
 * The two data-movement steps on their own (App. C, lowering phase, and its transpose), in the
 * canonical layout D-hat row-major [C*kh*kw][ld], row (c*kh+ky)*kw+kx, column (n*Ho+oy)*Wo+ox,
 * ld >= N*Ho*Wo (columns beyond N*Ho*Wo are written as zero by omni_lower and ignored by
 * omni_col2im).  Lowering is a pure copy: every entry is bit-identical to an element of X or +0.
 * col2im adds, for each pixel, its contributing entries in ascending (ky, kx) order in fp32.
 */
int omni_lower(const omni_conv_desc *desc, const void *X, void *Dhat, int64_t ld, void *hip_stream);
int omni_col2im(const omni_conv_desc *desc, const void *dDhat, int64_t ld, void *dX,
                void *hip_stream);

/*
 * Layers between the convolutions of the paper's networks (named in App. C, "Data Parallelism in
 * non-GEMM Kernels").  `dtype` is an omni_dtype; `count` is in elements.
 *   relu_forward : y = max(0, x)                      (in place allowed)
 *   relu_backward: dx = (y > 0) ? dy : 0, y being the ReLU's output (or input)   (in place allowed)
 *   maxpool_forward : k x k window, stride s, no padding, over `planes` = N*C planes of H x W;
 *       ceil_mode != 0 keeps a last border-clipped window.  The first maximum in (ky, kx) scan
 *       order wins.  argmax (uint8 per output, nullable) receives ky*k+kx of the winner.
 *   maxpool_backward: dx [planes][H][W] (overwritten) receives each dy at its window's winner.
 *   maxpool_relu_backward: the same, times the gradient of a ReLU applied just before the pool, in one
 *       pass.  y_pooled [planes][Ho][Wo] is the forward pool's output: it equals the winner's value, so a
 *       window routes its gradient iff y_pooled > 0 (the result equals pool backward followed by
 *       dx = 0 where the pool's input <= 0, without reading that input).
 * omni_pool_output_dim is host only and returns the pooled extent or a negative status.
 */
int omni_relu_forward(int32_t dtype, int64_t count, const void *x, void *y, void *hip_stream);
int omni_relu_backward(int32_t dtype, int64_t count, const void *y, const void *dy, void *dx,
                       void *hip_stream);
int omni_pool_output_dim(int32_t in, int32_t k, int32_t stride, int32_t ceil_mode);
int omni_maxpool_forward(int32_t dtype, int64_t planes, int32_t H, int32_t W, int32_t k,
                         int32_t stride, int32_t ceil_mode, const void *x, void *y, uint8_t *argmax,
                         void *hip_stream);
int omni_maxpool_backward(int32_t dtype, int64_t planes, int32_t H, int32_t W, int32_t k,
                          int32_t stride, int32_t ceil_mode, const void *dy, const uint8_t *argmax,
                          void *dx, void *hip_stream);
int omni_maxpool_relu_backward(int32_t dtype, int64_t planes, int32_t H, int32_t W, int32_t k,
                               int32_t stride, int32_t ceil_mode, const void *dy, const uint8_t *argmax,
                               const void *y_pooled, void *dx, void *hip_stream);

/*
 * The output gradient in the form the model gradient multiplies (Sec. III-B: the batch's output as ONE matrix whose
 * columns run over all images' positions; Sec. II-B: its gradient is the left operand of the model-gradient product).
 * With OMNI_FLAG_FUSED, bf16, the model gradient of the same-size stride-1 layers reads dY as the "rows" matrix
 *     dY_rows [F][ld] bf16:  dY_rows[f][n * plane_pitch + j] = dY[n][f][j],  j < Ho*Wo;  zero for Ho*Wo <= j < plane_pitch,
 * which omni_conv_backward_weights writes into its workspace on every call.  The layer that PRODUCES dY (the ReLU
 * and/or pooling layer behind the convolution) can write that form directly, and both backward passes read it:
 *   omni_conv_dy_rows_layout: ld and plane_pitch (elements) for this layer, plane_pitch = Ho*Wo rounded up to 8 and
 *       ld = N * plane_pitch; OMNI_UNSUPPORTED when the layer's model gradient does not read the rows form (then the
 *       plain entry points are the ones to call).  Host only.
 *   omni_relu_backward_rows: dx_rows = rows form of (y > 0 ? dy : 0) for dense y, dy [N][C][plane] (bf16, 8 <= plane
 *       <= 2048, C <= 65535; ld a multiple of 8, >= N * (plane rounded up to 8)); plane_sums (nullable) is fp32
 *       [C][N] and receives the sum of every plane's stored values -- the partial sums of the bias gradient.
 *   omni_maxpool_backward_rows: omni_maxpool_backward (y == NULL) or omni_maxpool_relu_backward (y = the pooled
 *       values) writing dx in the rows form of the [N][C][H][W] gradient, same plane_sums; bf16, 3 x 3 windows at
 *       stride 2 on planes of at most about 100 x 100, OMNI_UNSUPPORTED otherwise.
 *   omni_conv_backward_weights_rows: omni_conv_backward_weights reading dY_rows (not modified); dbias, if wanted, is
 *       the ordered sum of the partial sums plane_sums [F][sums_per_filter] (any partition of a filter's row of
 *       dY_rows into partial sums: the producers' N plane sums, or the column sums of the call below), which must
 *       then be given.  dW is bit-identical to the plain entry point's.  Workspace as for OMNI_PASS_BACKWARD_WEIGHTS.
 *   omni_conv_backward_data_rows: omni_conv_backward_data_packed reading dY_rows; dX is bit-identical.  Workspace as
 *       for OMNI_PASS_BACKWARD_DATA.
 *   omni_conv_backward_data_relu_rows: the same data gradient when the layer in front is convolution + ReLU with
 *       nothing between: its result dX [N][C][H][W] IS that layer's output gradient once the ReLU's mask is applied,
 *       so it is stored as dX_rows [C][ld_out] = rows form of (y_front > 0 ? dX : 0), y_front [N][C][H][W] (bf16)
 *       being the front layer's output; ld_out a multiple of 8, >= N * (H*W rounded up to 8).  Only the planes'
 *       H*W real columns are written: the round-up columns must be zero already (zero the buffer once).  col_sums
 *       (nullable) is fp32 [C][sums_per_channel] and receives partial sums of every row's stored values
 *       (sums_per_channel from omni_conv_backward_data_relu_rows_sums, host only; OMNI_UNSUPPORTED when this layer's
 *       data gradient cannot store this way, e.g. at batches so small that its reduction is split).
 * Columns of dx_rows beyond N * plane_pitch are never written.  All pointers 16-byte aligned.
 */
int omni_conv_dy_rows_layout(const omni_conv_desc *desc, int64_t *ld, int64_t *plane_pitch);
int omni_relu_backward_rows(int32_t dtype, int32_t N, int32_t C, int64_t plane, const void *y, const void *dy,
                            void *dx_rows, int64_t ld, float *plane_sums, void *hip_stream);
int omni_maxpool_backward_rows(int32_t dtype, int32_t N, int32_t C, int32_t H, int32_t W, int32_t k, int32_t stride,
                               int32_t ceil_mode, const void *dy, const uint8_t *argmax, const void *y, void *dx_rows,
                               int64_t ld, float *plane_sums, void *hip_stream);
int omni_conv_backward_weights_rows(const omni_conv_desc *desc, const void *X, const void *dY_rows,
                                    const float *plane_sums, int32_t sums_per_filter, float *dW, float *dbias,
                                    void *workspace, size_t workspace_bytes, void *hip_stream);
int omni_conv_backward_data_rows(const omni_conv_desc *desc, const void *dY_rows, const void *packed, void *dX,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);
int omni_conv_backward_data_relu_rows_sums(const omni_conv_desc *desc, int32_t *sums_per_channel);
int omni_conv_backward_data_relu_rows(const omni_conv_desc *desc, const void *dY_rows, const void *packed,
                                      const void *y_front, void *dX_rows, int64_t ld_out, float *col_sums,
                                      void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Normalisation across channels and dropout: the other two non-GEMM layers of the paper's CaffeNet runs (App. C,
 * "Data Parallelism in non-GEMM Kernels" names them beside pooling and ReLU; the paper prints no formula, the
 * definitions are those of the AlexNet network it trains, in the convention of the framework it matches layer by
 * layer).  x, y, dy, dx are [N][C][plane] (plane = H*W) of `dtype`.
 *   lrn_forward : s = k + (alpha / size) * sum_{|c' - c| <= size/2, 0 <= c' < C} x[n,c',p]^2;  y = x * s^(-beta).
 *       size odd, at most 9 (OMNI_UNSUPPORTED otherwise).  scale (nullable, fp32 [N][C][plane]) receives s; the
 *       backward pass needs it.  Arithmetic in fp32, one rounding on store.
 *   lrn_backward: dx = dy * s^(-beta) - (2 alpha beta / size) * x * sum_{|c' - c| <= size/2} dy[c'] x[c'] s[c']^(-beta-1).
 *   dropout_forward : y[i] = keep(i) ? x[i] / (1 - p) : 0, 0 <= p < 1.  keep(i) comes from the counter-based
 *       generator Philox4x64-10: block i / 8 (counter {i / 8, 0, 0, 0}, key {seed, stream_id}) yields four 64-bit
 *       words = eight 32-bit draws, low half first; element i is kept iff draw i mod 8 >= floor(p * 2^32).  No mask
 *       is stored: dropout_backward (dx[i] = keep(i) ? dy[i] / (1 - p) : 0) regenerates it from the same
 *       (p, seed, stream_id).  In place allowed.
 */
int omni_lrn_forward(int32_t dtype, int64_t N, int32_t C, int64_t plane, int32_t size, float alpha, float beta,
                     float k, const void *x, void *y, float *scale, void *hip_stream);
int omni_lrn_backward(int32_t dtype, int64_t N, int32_t C, int64_t plane, int32_t size, float alpha, float beta,
                      float k, const void *x, const void *dy, const float *scale, void *dx, void *hip_stream);
int omni_dropout_forward(int32_t dtype, int64_t count, float p, uint64_t seed, uint64_t stream_id,
                         const void *x, void *y, void *hip_stream);
int omni_dropout_backward(int32_t dtype, int64_t count, float p, uint64_t seed, uint64_t stream_id,
                          const void *dy, void *dx, void *hip_stream);

/*
 * Per-kernel timing (the paper times with a wall clock, App. C "Experiment Setup"; on a GPU the
 * equivalent is an event pair on the stream).  omni_profile_enable(1) clears earlier records and
 * makes every later launch of the library record a start and a stop event on its stream, tagged
 * with a kernel class and that launch's algorithmic work; omni_profile_enable(0) stops recording
 * and clears.  omni_profile_summary waits for the recorded events of one kernel class and returns
 * the number of launches, their summed duration in milliseconds, and their summed algorithmic
 * flops (GEMMs: 2*M*K*F) and bytes (data-movement kernels: each operand read or written once).
 * Kernel classes are numbered 0 .. omni_profile_kernel_count()-1 and named by
 * omni_profile_kernel_name.  omni_profile_select(k) restricts recording to kernel class k (the two events
 * around a launch cost a few microseconds of stream time each, which adds up over a step's ~50 launches);
 * -1 records all again, and so does every omni_profile_enable call.  omni_profile_select_mask records the
 * classes whose bit (1 << kernel class) is set, e.g. all matrix-core classes.  Host memory only; not
 * thread-safe against concurrent launches.
 */
int omni_profile_enable(int on);
int omni_profile_select(int kernel_id);
int omni_profile_select_mask(uint64_t mask);
int omni_profile_kernel_count(void);
const char *omni_profile_kernel_name(int kernel_id);
int omni_profile_summary(int kernel_id, int64_t *launches, double *total_ms, double *flops,
                         double *bytes);

/*
 * Tile overrides for tuning sweeps and tests -- not for production callers: the library chooses its tiles from
 * the layer's shape.  Process-wide, host only, not thread-safe against concurrent calls.
 *   OMNI_TUNE_GEMM_TILE: index of the GEMM tile configuration (-1: choose)
 *   OMNI_TUNE_FUSED_BN : column tile of the fused convolution: 256, 384 or 512 (0: choose)
 *   OMNI_TUNE_FUSED_BM : row tile of the fused convolution: 96 or 128 (0: choose)
 *   OMNI_TUNE_FUSED_PITCH : 1 keeps the fused convolution's LDS patch at the bare padded row width, 0 lets it take the
 *                           pitch that keeps fragment reads free of bank conflicts where the patch still fits
 *   OMNI_TUNE_WGRAD_SPLITS: most ranges the LDS-patch model gradients split their reduction into (0: choose)
 *   OMNI_TUNE_WGRAD_PATCH : 1 switches the LDS-patch model gradients off (their layers take the direct loader), 0 on
 *   OMNI_TUNE_POOL_LDS    : 1 sends the bf16 3 x 3 / stride 2 pools through the kernels that stage planes in LDS, 0 lets
 *                           them take the kernels that read the planes directly
 * An override that does not fit a layer is ignored for that layer.
 */
enum { OMNI_TUNE_GEMM_TILE = 0, OMNI_TUNE_FUSED_BN = 1, OMNI_TUNE_FUSED_BM = 2, OMNI_TUNE_WGRAD_SPLITS = 3, OMNI_TUNE_WGRAD_PATCH = 4,
       OMNI_TUNE_FUSED_PITCH = 5, OMNI_TUNE_POOL_LDS = 6 };
int omni_tuning_set(int knob, int value);

/* Host only.  Static string for a status code. */
const char *omni_status_string(int status);

/* Host only.  Library version, "major.minor". */
const char *omni_version(void);

#ifdef __cplusplus
}
#endif
#endif /* OMNICONV_H */

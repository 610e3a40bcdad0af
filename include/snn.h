/*
 * snn.h - C ABI of the MI355X (gfx950) sub-bit binary 3x3 convolution library.
 *
 * The library implements the inference/forward hot path of "Sub-bit Neural Networks"
 * (arXiv 2110.09195): a 3x3 convolution whose +-1 kernels are members of a small per-layer
 * subset P (the "codebook", K = 2^tau binary 3x3 kernels out of 512) addressed by an index
 * per (output channel, input channel) pair, evaluated in the two stages of Sec. 4.5 / Fig. 6
 * (each input channel is convolved once with each of the K kernels; each output channel then
 * gathers the pre-computed responses by index and sums them along c_in), plus the 1-bit
 * XNOR/popcount convolution it is compared with (Sec. 3), the sign/bit-packing of
 * activations (Alg. 1 forward) and the nearest-subset-member projection (Eq. 2 / Eq. 5).
 * Around these: the convolution ending in the next layer's sign (1-bit activations from layer to
 * layer), the training-side lines of Alg. 1 (Eq. 3, Eq. 4, the gradient of the subset), the
 * tau-bit index storage of Sec. 4.4, the extension to 1x1 layers (appendix) and, as a yardstick, the
 * same layers as dense contractions on the matrix cores.
 *
 * General rules for every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller (hipMalloc / a torch CUDA
 *     tensor's data_ptr).  Descriptor structs are HOST pointers, read before the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Every call only
 *     enqueues work on that stream and returns without synchronising.
 *   - The library never allocates, frees or keeps device memory; scratch space is the
 *     caller's `workspace` (size from snn_workspace_bytes), used only during the call -
 *     except between a *_prepare call and the *_prepared calls that follow it, which read
 *     what the preparation left there.  Two calls that share a workspace must be ordered
 *     (same stream, or synchronised).
 *   - Return value: SNN_OK (0) or a negative SNN_ERR_* code.  On error nothing has been
 *     enqueued.  No exceptions, no aborts, nothing printed.
 *   - Values of idx[] must be < K and values of codebook[] / w9[] must be < 512; this is
 *     not reported by the device: the table-building kernels read an index >= K as K - 1 and
 *     mask a code to 9 bits, so that only memory inside the library's own tables is ever read
 *     with them; the result for such input is that of the clamped value, with no error.
 *
 * Conventions (identical in the CPU oracle the library is tested against)
 *   - Kernel code (Sec. 4.1): a binary 3x3 kernel is flattened row-major, +1 -> bit 1,
 *     -1 -> bit 0, first element most significant.  code = paper index - 1, so 0 is the
 *     all(-1) kernel and 511 the all(+1) kernel.  Tap t = 3*dy + dx is bit (8 - t).
 *   - Convolution (Sec. 3): cross-correlation (no kernel flip), 3x3, zero padding 1,
 *     stride 1 or 2, H_out = (H - 1) / stride + 1, no bias.  Taps that fall outside the
 *     image contribute 0, also for +-1 activations.
 *   - Activation sign (Alg. 1 forward): x >= 0 -> +1 (bit 1), otherwise -1 (bit 0); NaN -> -1.
 *   - Output: fp32 NCHW, y[n][co][ho][wo] = (float)S * alpha[co] for +-1 activations (S the
 *     exact integer sum, one fp32 multiply) and alpha[co] * S with S accumulated in fp32 for
 *     fp32 activations.
 */
#ifndef SNN_H
#define SNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* status codes */
#define SNN_OK               0
#define SNN_ERR_INVALID_ARG (-1)  /* null pointer, non-positive size, K outside 1..512, bad enum */
#define SNN_ERR_UNSUPPORTED (-2)  /* a valid request this build has no kernel for (listed per call) */
#define SNN_ERR_WORKSPACE   (-3)  /* workspace null, misaligned or ws_bytes too small */
#define SNN_ERR_LAUNCH      (-4)  /* the HIP runtime refused a launch */

/* activation layouts (snn_conv_desc.act and the `layout` argument of snn_pack_activations) */
#define SNN_ACT_BIN_ROWS     0    /* uint32 [N][C][H][ceil(W/32)], bit (w % 32) of word (w / 32) */
#define SNN_ACT_BIN_CHANNELS 1    /* uint32 [N][H][W][ceil(C/32)], bit (c % 32) of word (c / 32) */
#define SNN_ACT_F32          2    /* float  [N][C][H][W] (weight-only variant, W/A = x/32)       */
/* In both packed layouts bit 1 means +1, and the unused high bits of a last word are 0. */

/* which entry point a workspace is for */
#define SNN_WS_SUBBIT 0
#define SNN_WS_BNN    1
#define SNN_WS_FORWARD 2
#define SNN_WS_CONV1X1 3
#define SNN_WS_BNN_DENSE 4

/* One 3x3 layer (Sec. 3 notation: c_in, c_out, H, W of the input). */
typedef struct snn_conv_desc {
    int32_t N;       /* batch                                   */
    int32_t C_in;    /* input channels  (1 .. 4096)             */
    int32_t C_out;   /* output channels (>= 1)                  */
    int32_t H, W;    /* input height and width                  */
    int32_t stride;  /* 1 or 2                                  */
    int32_t K;       /* subset size 1 .. 512 (ignored by snn_bnn_conv2d) */
    int32_t act;     /* SNN_ACT_*                               */
} snn_conv_desc;

/*
 * Alg. 1 forward, sign(a^{i-1}): binarise fp32 activations and pack them 32 per word.
 *   x_nchw  device, float [N][C][H][W]
 *   packed  device, snn_packed_bytes(N, C, H, W, layout) bytes, layout SNN_ACT_BIN_ROWS or
 *           SNN_ACT_BIN_CHANNELS; fully overwritten.
 * Errors: INVALID_ARG (null pointers, sizes < 1, layout not one of the two packed ones).
 */
int snn_pack_activations(const float *x_nchw, void *packed, int N, int C, int H, int W,
                         int layout, void *stream);

/*
 * snn_pack_activations for several tensors at once: the packed-rows items share launches (32 tensors each),
 * packed-channels items get a launch of their own.  Results are those of one snn_pack_activations call per item.
 * (The inputs of a stack of layers are mostly smaller than what the chip moves while a launch starts and drains.)
 *   items[i].x_nchw  device, float [N][C][H][W];   items[i].packed  device, the packed tensor in items[i].layout
 * Errors: INVALID_ARG (any item; nothing is enqueued); LAUNCH.
 */
typedef struct snn_pack_item {
    const float *x_nchw;
    void *packed;
    int32_t N, C, H, W;
    int32_t layout;
} snn_pack_item;
int snn_pack_activations_many(const snn_pack_item *items, int n_items, void *stream);

/*
 * Eq. 2 / Eq. 5 / Alg. 1 forward: for each real-valued 3x3 kernel, the index of the nearest
 * member of the subset, arg min_k ||P_k - w||^2 = arg max_k <P_k, w> (all members have the
 * same norm).  The inner product is accumulated in fp32 from 0 over taps 0..8 in order,
 * adding w_t where the member's tap is +1 and subtracting it where it is -1; among equal
 * scores the lowest index wins.
 *   w         device, float [n][9] (row-major 3x3 kernels, any (c_out, c_in) order)
 *   codebook  device, uint16 [K], 9-bit codes (distinct, as Sec. 4.3 requires; duplicates
 *             are harmless: the lower index is returned)
 *   idx_out   device, uint16 [n]
 * n = 0 is allowed and does nothing.  Errors: INVALID_ARG.
 */
int snn_project_kernels(const float *w, int64_t n, const uint16_t *codebook, int K,
                        uint16_t *idx_out, void *stream);

/*
 * Sec. 4.5 / Fig. 6: the sub-bit convolution.  Stage 1 convolves every input channel with the
 * K subset kernels (responses stay on chip), stage 2 sums, for each output channel, the
 * responses its indices select; then y = alpha * S.
 *   desc      host; act = SNN_ACT_BIN_ROWS (+-1 activations) or SNN_ACT_F32
 *   x         device, activations in the layout desc->act names
 *   codebook  device, uint16 [K] 9-bit codes
 *   idx       device, uint16 [C_out][C_in], values < K
 *   alpha     device, float [C_out]   (the paper's channel-wise lambda)
 *   y_nchw    device, float [N][C_out][H_out][W_out], fully overwritten
 *   workspace device, >= snn_workspace_bytes(desc, SNN_WS_SUBBIT) bytes, 256-byte aligned
 * Errors: INVALID_ARG; UNSUPPORTED for act = SNN_ACT_BIN_CHANNELS (pack rows instead) and for
 * packed inputs of 2^31 words (8 GiB) or more; WORKSPACE; LAUNCH.
 */
int snn_subbit_conv2d(const snn_conv_desc *desc, const void *x, const uint16_t *codebook,
                      const uint16_t *idx, const float *alpha, float *y_nchw,
                      void *workspace, size_t ws_bytes, void *stream);

/*
 * snn_subbit_conv2d for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results
 * and errors as snn_subbit_conv2d, without `workspace` / `ws_bytes`: the tables the call builds live
 * in a buffer inside the library, SNN_NOALLOC_MAX_WORKSPACE_BYTES per GPU, held until the process
 * ends.  The call allocates and frees nothing.  A layer whose tables need more
 * (snn_workspace_bytes(desc, SNN_WS_SUBBIT) > SNN_NOALLOC_MAX_WORKSPACE_BYTES) is refused with
 * SNN_ERR_WORKSPACE and nothing is enqueued; SNN_ERR_LAUNCH also if the buffer's address cannot be
 * obtained.  All calls on one GPU share the buffer: every call rebuilds what it reads, and calls
 * that overlap on one GPU (different streams, or threads) race - issue them on one stream.
 */
#define SNN_NOALLOC_MAX_WORKSPACE_BYTES (4 * 1024 * 1024)
int snn_subbit_conv2d_noalloc(const snn_conv_desc *desc, const void *x, const uint16_t *codebook,
                              const uint16_t *idx, const float *alpha, float *y_nchw, void *stream);

/*
 * snn_subbit_conv2d in two halves, for weights that stay fixed over many calls (inference):
 * snn_subbit_prepare turns codebook, idx and alpha into the tables the convolution reads (one small
 * launch; to be repeated whenever one of them changes), snn_subbit_conv2d_prepared is the
 * convolution alone (one launch).  prepare followed by conv2d_prepared on the same stream equals
 * snn_subbit_conv2d bit for bit.  The environment overrides that select kernels must not change
 * between the two calls.
 *   workspace  the same buffer in both calls (>= snn_workspace_bytes(desc, SNN_WS_SUBBIT) bytes,
 *              256-byte aligned); its contents belong to the library until the weights change
 *   alpha      the same values in both calls (some kernels read alpha at convolution time)
 *   everything else as for snn_subbit_conv2d, same errors.
 */
int snn_subbit_prepare(const snn_conv_desc *desc, const uint16_t *codebook, const uint16_t *idx,
                       const float *alpha, void *workspace, size_t ws_bytes, void *stream);
int snn_subbit_conv2d_prepared(const snn_conv_desc *desc, const void *x, const float *alpha,
                               float *y_nchw, void *workspace, size_t ws_bytes, void *stream);

/*
 * Sec. 4.4 / Fig. 5: the storage format of a sub-bit layer, tau bits per kernel (tau / 9 bit per
 * weight).  Index i occupies bits [i * tau, (i + 1) * tau) of a little-endian bit stream of 32-bit
 * words (bit b of the stream is bit b % 32 of word b / 32); unused high bits of the last word are 0.
 *   snn_packed_index_bytes(n, tau)   bytes of the stream for n indices (0 for invalid arguments); host-only
 *   snn_pack_indices                 idx uint16 [n] (values < 2^tau) -> packed, tau in 1..9
 *   snn_subbit_prepare_packed        snn_subbit_prepare reading the stream directly (the indices are
 *                                    unpacked inside the preparation kernel); follow with
 *                                    snn_subbit_conv2d_prepared.  desc->K <= 2^tau; +-1 activations and the
 *                                    matrix-core kernel only (K <= 64), else UNSUPPORTED.
 */
size_t snn_packed_index_bytes(int64_t n, int tau);
int snn_pack_indices(const uint16_t *idx, int64_t n, int tau, void *packed, void *stream);
int snn_subbit_prepare_packed(const snn_conv_desc *desc, const uint16_t *codebook, const void *idx_packed,
                              int tau, const float *alpha, void *workspace, size_t ws_bytes, void *stream);

/*
 * Alg. 1 forward of one layer in one call: the projection of the layer's real-valued kernels
 * (Eq. 2 / Eq. 5), sign(a) of its fp32 input, and the sub-bit convolution (Sec. 4.5 / Fig. 6) of
 * the two.  idx_out and y_nchw equal, bit for bit, what snn_project_kernels,
 * snn_pack_activations(SNN_ACT_BIN_ROWS) and snn_subbit_conv2d produce one after the other;
 * the small operations share one launch, so the call costs two launches instead of four.
 *   desc      host; act must be SNN_ACT_BIN_ROWS (+-1 activations; the packed rows live in the
 *             workspace)
 *   x_nchw    device, float [N][C_in][H][W]
 *   w         device, float [C_out][C_in][9] (row-major 3x3 kernels)
 *   codebook  device, uint16 [K] 9-bit codes
 *   alpha     device, float [C_out]
 *   idx_out   device, uint16 [C_out][C_in], fully overwritten (the projection, which a backward
 *             pass needs again)
 *   y_nchw    device, float [N][C_out][H_out][W_out], fully overwritten
 *   workspace device, >= snn_workspace_bytes(desc, SNN_WS_FORWARD) bytes, 256-byte aligned
 * Errors: INVALID_ARG; UNSUPPORTED for any other desc->act and for packed inputs of 2^31 words
 * or more; WORKSPACE; LAUNCH.
 */
int snn_subbit_forward(const snn_conv_desc *desc, const float *x_nchw, const float *w,
                       const uint16_t *codebook, const float *alpha, uint16_t *idx_out,
                       float *y_nchw, void *workspace, size_t ws_bytes, void *stream);

/*
 * The sub-bit convolution (Sec. 4.5) followed by the next layer's binarisation (Alg. 1 forward:
 * sign(a^i), after the channel-wise affine that batch normalisation folds into alpha and beta):
 *   bit[n][co][ho][wo] = ( fl(fl((float)S * alpha[co]) + beta[co]) >= 0 )
 * with S the integer convolution sum and fl() rounding to fp32 (no fused multiply-add), written
 * as packed rows, the layout snn_subbit_conv2d consumes: a stack of layers passes 1-bit
 * activations from layer to layer and never writes fp32 activations.
 *   desc       host; act must be SNN_ACT_BIN_ROWS
 *   x_packed   device, uint32 [N][C_in][H][ceil(W/32)]
 *   codebook, idx, alpha: as for snn_subbit_conv2d;  beta  device, float [C_out]
 *   out_packed device, uint32 [N][C_out][H_out][ceil(W_out/32)], fully overwritten (unused high
 *              bits of a last word 0)
 *   workspace  device, >= snn_workspace_bytes(desc, SNN_WS_SUBBIT) bytes, 256-byte aligned
 * Errors: INVALID_ARG; UNSUPPORTED for any other desc->act and for layers outside the
 * matrix-core kernel (K > 64, or C_in = 1 with K <= 32, or tensors of 2^30 words or more);
 * WORKSPACE; LAUNCH.
 */
int snn_subbit_conv2d_sign(const snn_conv_desc *desc, const void *x_packed, const uint16_t *codebook,
                           const uint16_t *idx, const float *alpha, const float *beta,
                           void *out_packed, void *workspace, size_t ws_bytes, void *stream);

/*
 * snn_subbit_conv2d_sign in two halves for fixed weights, like snn_subbit_prepare /
 * snn_subbit_conv2d_prepared: the tables (thresholds included) once, then one launch per call.
 * A stack of prepared layers runs with one launch per layer and 1-bit activations throughout.
 * The workspace of snn_subbit_prepare_sign serves only snn_subbit_conv2d_sign_prepared (and
 * that of snn_subbit_prepare only snn_subbit_conv2d_prepared).
 */
int snn_subbit_prepare_sign(const snn_conv_desc *desc, const uint16_t *codebook, const uint16_t *idx,
                            const float *alpha, const float *beta, void *workspace, size_t ws_bytes,
                            void *stream);
int snn_subbit_conv2d_sign_prepared(const snn_conv_desc *desc, const void *x_packed, void *out_packed,
                                    void *workspace, size_t ws_bytes, void *stream);

/*
 * The weights-side work of a whole stack of layers in ONE launch: for every layer the projection of
 * its real-valued kernels (Eq. 2 / Eq. 5; idx_out as snn_project_kernels writes it) and the tables
 * of snn_subbit_prepare (beta == NULL; follow with snn_subbit_conv2d_prepared) or of
 * snn_subbit_prepare_sign (beta given; follow with snn_subbit_conv2d_sign_prepared).  A training
 * step's forward pass is then this call plus, per layer, the packing (where the input is fp32) and
 * one convolution launch.
 *   layers    host array of n_layers entries (read during the call only); all pointers inside are
 *             device pointers with the meanings and sizes of the single-layer calls; desc.act must be
 *             SNN_ACT_BIN_ROWS; workspace: SNN_WS_SUBBIT bytes, 256-byte aligned, one per layer
 * Errors: INVALID_ARG; UNSUPPORTED if some layer is outside the matrix-core kernel (K > 64, or
 * C_in = 1 with K <= 32); WORKSPACE; LAUNCH.  On error nothing is enqueued.
 */
typedef struct snn_layer_weights {
    snn_conv_desc desc;
    const float *w;            /* [C_out][C_in][9] */
    const uint16_t *codebook;  /* [K] */
    const float *alpha;        /* [C_out] */
    const float *beta;         /* [C_out], or NULL for the fp32 output */
    uint16_t *idx_out;         /* [C_out][C_in] */
    void *workspace;
    size_t ws_bytes;
} snn_layer_weights;
int snn_subbit_project_prepare_many(const snn_layer_weights *layers, int n_layers, void *stream);

/*
 * snn_subbit_conv2d_prepared for several layers that do not depend on each other (each reads its own
 * input), e.g. the 3x3 layers of a network whose inputs are all resident: the two stages of Sec. 4.5
 * for every layer, as few launches as possible (layers whose form the shared kernel holds go
 * sixteen to a launch, any other layer gets a launch of its own).  The results are those of one
 * snn_subbit_conv2d_prepared call per layer, bit for bit; what changes is that the layers share the
 * chip instead of each ending with a few busy compute units.
 *   layers[l].desc       host; act must be SNN_ACT_BIN_ROWS, K <= 64 (C_in >= 2 if K <= 32)
 *   layers[l].x_packed   device, packed rows of the layer's input
 *   layers[l].y_nchw     device, float [N][C_out][H_out][W_out], fully overwritten; the outputs of
 *                        different layers must not overlap
 *   layers[l].workspace  device, as prepared by snn_subbit_prepare / snn_subbit_prepare_packed /
 *                        snn_subbit_project_prepare_many (beta == NULL) for the same desc.  The tables
 *                        are only read.  The scheduling words at the end of layers[0].workspace (zero after
 *                        preparation) count work items while the call runs and are zero again when it
 *                        ends: calls that share that workspace must be ordered, like any two calls that
 *                        share a workspace.
 * Errors: INVALID_ARG; UNSUPPORTED (a layer outside the matrix-core kernel); WORKSPACE; LAUNCH.  All
 * layers are checked before anything is enqueued.
 */
typedef struct snn_layer_io {
    snn_conv_desc desc;
    const void *x_packed;
    float *y_nchw;
    void *workspace;
    size_t ws_bytes;
} snn_layer_io;
int snn_subbit_conv2d_prepared_many(const snn_layer_io *layers, int n_layers, void *stream);

/*
 * Alg. 1 forward of a whole stack of independent layers in THREE launches: one binarises and packs every
 * layer's fp32 input (snn_pack_activations_many), one projects every layer's real-valued kernels onto its subset
 * (Eq. 2 / Eq. 5) and builds the convolution's tables (snn_subbit_project_prepare_many), the third is the launch
 * of snn_subbit_conv2d_prepared_many over all layers.  (The first two are independent: a caller with two streams
 * can issue these three calls itself and overlap them.)
 * Results (idx_out, y_nchw) are those of one snn_subbit_forward call per layer, bit for bit.
 *   layers[l].desc       host; act must be SNN_ACT_BIN_ROWS, K <= 64 (C_in >= 2 if K <= 32)
 *   layers[l].x_nchw     device, float [N][C_in][H][W]
 *   layers[l].w          device, float [C_out][C_in][9];   codebook  device, uint16 [K];   alpha  device, float [C_out]
 *   layers[l].idx_out    device, uint16 [C_out][C_in], fully overwritten
 *   layers[l].y_nchw     device, float [N][C_out][H_out][W_out], fully overwritten; outputs must not overlap
 *   layers[l].workspace  device, >= snn_workspace_bytes(desc, SNN_WS_FORWARD) bytes, 256-byte aligned, one per layer;
 *                        afterwards it holds the layer's tables and packed input (usable by the *_prepared calls)
 * Errors: INVALID_ARG; UNSUPPORTED (a layer outside the matrix-core kernel); WORKSPACE; LAUNCH.  All layers are
 * checked before anything is enqueued.
 */
typedef struct snn_layer_forward {
    snn_conv_desc desc;
    const float *x_nchw;
    const float *w;
    const uint16_t *codebook;
    const float *alpha;
    uint16_t *idx_out;
    float *y_nchw;
    void *workspace;
    size_t ws_bytes;
} snn_layer_forward;
int snn_subbit_forward_many(const snn_layer_forward *layers, int n_layers, void *stream);

/*
 * The same with the projection of the layer's real-valued kernels in front (Alg. 1 forward of a
 * layer inside a stack): idx_out = project(w) as snn_project_kernels computes it, then
 * snn_subbit_conv2d_sign with it; two launches.
 *   w        device, float [C_out][C_in][9];  idx_out  device, uint16 [C_out][C_in], fully overwritten
 *   the rest as for snn_subbit_conv2d_sign (workspace: SNN_WS_SUBBIT).
 */
int snn_subbit_forward_sign(const snn_conv_desc *desc, const void *x_packed, const float *w,
                            const uint16_t *codebook, const float *alpha, const float *beta,
                            uint16_t *idx_out, void *out_packed, void *workspace, size_t ws_bytes,
                            void *stream);

/*
 * Alg. 1 backward, the two lines that touch the kernels of a layer.  Given the gradient w.r.t. the
 * binarised kernels w_bar (from the convolution's backward pass, which is not part of this library):
 *   g_w[c][t] = g_wbar[c][t] if -1 < w[c][t] < 1 else 0       (Eq. 3, straight-through estimator, per element)
 *   g_p[k][t] = sum over the kernels c with idx[c] == k of g_wbar[c][t]
 *               (the gradient of the subset tensor p, taken as that of its sign memory m:
 *                backward of Eq. 5 / the p-update of Alg. 1); summed in fp32, per block of 512
 *                kernels in unspecified order (LDS float atomics), the block sums then in a fixed
 *                order: g_p can differ in its last bits from run to run on the same input
 *   w, g_wbar  device, float [n][9];  idx  device, uint16 [n], values < K (as snn_project_kernels wrote them)
 *   g_w        device, float [n][9], fully overwritten;  g_p  device, float [K][9], fully overwritten
 *   workspace  device, >= snn_project_backward_workspace_bytes(n, K) bytes, 256-byte aligned
 * n = 0 is allowed (g_p = 0).  Errors: INVALID_ARG; WORKSPACE; LAUNCH.
 */
int snn_project_backward(const float *w, const float *g_wbar, const uint16_t *idx, int64_t n, int K,
                         float *g_w, float *g_p, void *workspace, size_t ws_bytes, void *stream);
size_t snn_project_backward_workspace_bytes(int64_t n, int K);

/*
 * Eq. 4 and the repeated-member check of Sec. 4.3, for one layer's subset:
 *   m[k][t]     <- sign(p[k][t]) where |p[k][t]| > theta, unchanged elsewhere      (m in {+1, -1})
 *   codebook[k]  = the 9-bit code of m[k] (tap t at bit 8 - t, +1 -> 1): the subset the next forward pass uses
 *   dup[k]       = 1 if some j < k has the same code (the caller replaces such members by freshly
 *                  sampled kernels; the random draw is the caller's), else 0
 *   p  device, float [K][9];  m  device, int8 [K][9], updated in place;  theta >= 0
 *   codebook_out  device, uint16 [K];  dup_out  device, uint8 [K]
 * Errors: INVALID_ARG (null pointers, K outside 1..512, theta negative or NaN); LAUNCH.
 */
int snn_subset_update(const float *p, int8_t *m, float theta, int K, uint16_t *codebook_out,
                      uint8_t *dup_out, void *stream);

/*
 * The extension to 1x1 layers (appendix "Extending to Bottleneck with 1x1 Kernels", Table 5): the
 * c_out x c_in weights are cut into vectors of 8 consecutive input channels, every vector is a
 * member of a layer-specific subset of {+-1}^8 (K = 2^tau' members, tau' / 8 bit per weight) and
 * is stored as its index.  Computed with the same sharing as the 3x3 layer: per pixel and group
 * of 8 channels the responses of the K members once, then per output channel the gather by
 * index and the sum over the c_in / 8 groups;  y = alpha * S, no padding, stride 1 or 2.
 *   desc       host; act must be SNN_ACT_BIN_CHANNELS (+-1 activations, 32 channels per word);
 *              C_in a multiple of 8; K <= 256 (this build: K <= 64, else UNSUPPORTED)
 *   x          device, uint32 [N][H][W][ceil(C_in/32)]
 *   codebook8  device, uint16 [K], 8-bit codes: element j of the vector (input channel 8 g + j) at
 *              bit 7 - j, +1 -> 1
 *   idx        device, uint16 [C_out][C_in / 8], values < K
 *   alpha, y_nchw: as for snn_subbit_conv2d;  H_out = floor((H - 1) / stride) + 1
 *   workspace  device, >= snn_workspace_bytes(desc, SNN_WS_CONV1X1) bytes, 256-byte aligned
 * Errors: INVALID_ARG; UNSUPPORTED (other desc->act, C_in not a multiple of 8, K > 64, or
 * C_in = 8 with K <= 32); WORKSPACE; LAUNCH.
 */
int snn_subbit_conv1x1(const snn_conv_desc *desc, const void *x, const uint16_t *codebook8,
                       const uint16_t *idx, const float *alpha, float *y_nchw, void *workspace,
                       size_t ws_bytes, void *stream);

/*
 * snn_subbit_conv1x1 in two halves for weights that stay fixed (inference): the first builds the layer's tables in
 * `workspace` (one small launch), the second is the convolution alone and may follow any number of times.  Same
 * arguments, results and errors as snn_subbit_conv1x1; the workspace must not be touched in between.
 */
int snn_subbit_conv1x1_prepare(const snn_conv_desc *desc, const uint16_t *codebook8, const uint16_t *idx,
                               const float *alpha, void *workspace, size_t ws_bytes, void *stream);
int snn_subbit_conv1x1_prepared(const snn_conv_desc *desc, const void *x, float *y_nchw, void *workspace,
                                size_t ws_bytes, void *stream);

/*
 * The projection of Eq. 2 / Eq. 5 for 1x1 layers (appendix, Table 5): for each real-valued vector
 * of 8 consecutive input-channel weights, the index of the nearest member of the layer's subset of
 * {+-1}^8, arg max_k <P'_k, w>, accumulated in fp32 from 0 over elements 0..7 in order (add where
 * the member's element is +1, subtract where it is -1); among equal scores the lowest index wins.
 *   w          device, float [n][8], 16-byte aligned (the c_out x c_in weights of a 1x1 layer
 *              row by row are exactly the [c_out * c_in / 8][8] vectors, in idx order)
 *   codebook8  device, uint16 [K], 8-bit codes (element j at bit 7 - j, +1 -> 1), 1 <= K <= 256
 *   idx_out    device, uint16 [n]
 * n = 0 is allowed and does nothing.  Errors: INVALID_ARG (also for a misaligned w).
 */
int snn_project_vectors8(const float *w, int64_t n, const uint16_t *codebook8, int K,
                         uint16_t *idx_out, void *stream);

/*
 * Sec. 3: the 1-bit layer a = lambda * (w_bar o a_bar), "o" = XNOR + bit count over words of
 * 32 input channels.  The baseline every sub-bit number is compared with.
 *   desc      host; act = SNN_ACT_BIN_CHANNELS (+-1 activations) or SNN_ACT_F32; K ignored
 *   x         device, activations in the layout desc->act names
 *   w9        device, uint16 [C_out][C_in], one 9-bit code per kernel
 *   alpha, y_nchw, workspace (SNN_WS_BNN), stream: as above
 * Errors: INVALID_ARG; UNSUPPORTED for act = SNN_ACT_BIN_ROWS and for packed inputs of 2^31
 * words (8 GiB) or more; WORKSPACE; LAUNCH.
 */
int snn_bnn_conv2d(const snn_conv_desc *desc, const void *x, const uint16_t *w9,
                   const float *alpha, float *y_nchw, void *workspace, size_t ws_bytes,
                   void *stream);

/*
 * snn_bnn_conv2d in two halves, for weights that stay fixed over many calls (the form the 1-bit layer of
 * Sec. 3 is timed in next to the prepared sub-bit calls): snn_bnn_prepare turns w9 into the bit planes
 * and border corrections the kernel reads (all that depends on the weights) and writes them to the
 * workspace; snn_bnn_conv2d_prepared runs the convolution from them.  Arguments as for snn_bnn_conv2d;
 * the workspace (SNN_WS_BNN) carries the prepared data between the two calls and must not be written in
 * between; the two calls together give exactly the result of snn_bnn_conv2d.  Same errors.
 */
int snn_bnn_prepare(const snn_conv_desc *desc, const uint16_t *w9, void *workspace, size_t ws_bytes, void *stream);
int snn_bnn_conv2d_prepared(const snn_conv_desc *desc, const void *x, const float *alpha, float *y_nchw,
                            void *workspace, size_t ws_bytes, void *stream);

/*
 * The same 1-bit layer (Sec. 3) evaluated as a dense contraction on the matrix cores instead of
 * XNOR + bit count: +-1 weights and activations as FP4 operands, zero for taps outside the
 * image, fp32 accumulation (exact: |S| <= 9 C_in < 2^24).  Results are identical to
 * snn_bnn_conv2d.  It is the dense yardstick of this chip for the cost model of Sec. 4.5: a
 * sub-bit layer expanded to its c_out x c_in kernels (w9[co][ci] = codebook[idx[co][ci]]) runs
 * through it unchanged.
 *   desc      host; act must be SNN_ACT_BIN_CHANNELS; K ignored
 *   x         device, uint32 [N][H][W][ceil(C_in/32)]
 *   w9        device, uint16 [C_out][C_in], one 9-bit code per kernel
 *   alpha, y_nchw, stream: as for snn_bnn_conv2d
 *   workspace device, >= snn_workspace_bytes(desc, SNN_WS_BNN_DENSE) bytes, 256-byte aligned
 *             (the weights in operand layout, rewritten by every call)
 * Errors: INVALID_ARG; UNSUPPORTED for any other desc->act, for packed inputs of 2^29 words
 * (2 GiB) or more and for 2^31 output pixels or more; WORKSPACE; LAUNCH.
 */
int snn_bnn_conv2d_dense(const snn_conv_desc *desc, const void *x, const uint16_t *w9,
                         const float *alpha, float *y_nchw, void *workspace, size_t ws_bytes,
                         void *stream);

/*
 * A sub-bit layer (Sec. 4.2: kernels given as indices into the layer's subset) through the same
 * dense contraction: the preparation kernel looks the kernels up (w9[co][ci] =
 * codebook[idx[co][ci]]) while it expands them.  Same results as snn_subbit_conv2d on the same
 * layer; the sharing of Sec. 4.5 is NOT used (it is the comparison point for it).
 *   desc      host; act must be SNN_ACT_BIN_CHANNELS; K = subset size
 *   codebook  device, uint16 [K];  idx  device, uint16 [C_out][C_in], values < K
 *   the rest as for snn_bnn_conv2d_dense (workspace: SNN_WS_BNN_DENSE).
 */
int snn_subbit_conv2d_dense(const snn_conv_desc *desc, const void *x, const uint16_t *codebook,
                            const uint16_t *idx, const float *alpha, float *y_nchw,
                            void *workspace, size_t ws_bytes, void *stream);

/*
 * The two halves of the dense calls for weights that stay fixed: snn_dense_prepare expands the
 * kernels into the workspace (codebook == NULL: `codes` are 9-bit kernel codes [C_out][C_in] and
 * desc->K is ignored; else `codes` are indices into codebook[K]); snn_dense_conv2d_prepared is
 * the contraction alone, one launch, any number of times.  The workspace (SNN_WS_BNN_DENSE bytes,
 * 256-byte aligned) belongs to the library between the two calls; together they give the same
 * result as the one-call forms.  Errors as for snn_bnn_conv2d_dense.
 */
int snn_dense_prepare(const snn_conv_desc *desc, const uint16_t *codebook, const uint16_t *codes,
                      void *workspace, size_t ws_bytes, void *stream);
int snn_dense_conv2d_prepared(const snn_conv_desc *desc, const void *x, const float *alpha,
                              float *y_nchw, void *workspace, size_t ws_bytes, void *stream);

/*
 * The prepared dense contraction ending in the next layer's binarisation (Alg. 1 forward,
 * sign(a^i), after the channel-wise affine alpha, beta; same definition as
 * snn_subbit_conv2d_sign): packed channels in, packed channels out, no fp32 activations.
 *   bit c % 32 of out[n][ho][wo][c / 32] = (fl(fl((float)S * alpha[c]) + beta[c]) >= 0)
 *   desc, x, alpha, workspace: as for snn_dense_conv2d_prepared (after snn_dense_prepare)
 *   beta        device, float [C_out]
 *   out_packed  device, uint32 [N][H_out][W_out][ceil(C_out/32)] (snn_packed_bytes(N, C_out,
 *               H_out, W_out, SNN_ACT_BIN_CHANNELS) bytes), fully overwritten, unused high bits 0:
 *               the input of the next layer's dense call as it is
 * Errors as for snn_dense_conv2d_prepared.
 */
int snn_dense_conv2d_sign_prepared(const snn_conv_desc *desc, const void *x, const float *alpha,
                                   const float *beta, void *out_packed, void *workspace,
                                   size_t ws_bytes, void *stream);

/* Bytes of workspace the given entry point (SNN_WS_*) needs for this layer; 0 if desc is
 * invalid or the combination is unsupported.  Host-only, no device work. */
size_t snn_workspace_bytes(const snn_conv_desc *desc, int which);

/* Bytes of a packed activation tensor in the given layout (also valid for SNN_ACT_F32);
 * 0 for invalid arguments.  Host-only. */
size_t snn_packed_bytes(int N, int C, int H, int W, int layout);

/* Static, human-readable name of a status code. */
const char *snn_status_string(int status);

/* Contraction slots per input channel that the matrix-core form of the sub-bit convolution spends on
 * this layer as launched (Sec. 4.5: the method needs one of them, the gather; the others multiply a zero
 * of the one-hot operand): 32 (two channels per matrix instruction, K <= 32), 16 (four channels,
 * K <= 16 on long channel runs), 64 (one channel, 32 < K <= 64); 0 where a kernel without matrix
 * instructions runs the layer (K > 64, C_in = 1, fp32 activations); negative SNN_ERR_* for an invalid desc.
 * Host-only; for the roofline accounting of a benchmark. */
int snn_subbit_slots_per_channel(const snn_conv_desc *desc);

/* Tuning and test switches.  Each knob holds SNN_TUNE_AUTO (the library's own choice) unless set; a knob's
 * first value is read ONCE, when the library first looks at any knob, from the environment variable named like
 * the knob without "TUNE_" (SNN_MFMA_TILE as "PB,CB").  They select among kernel forms that all compute the same result.
 * Table layouts in a workspace depend on them: a workspace written by a prepare call must be used under the
 * settings it was written under (not checked), and snn_workspace_bytes answers for the settings in force
 * when it is called.  Process-wide,
 * not synchronised with calls in flight on other threads.
 * snn_set_tuning returns SNN_ERR_INVALID_ARG for an unknown knob or a value outside the knob's list. */
#define SNN_TUNE_AUTO (-1)
#define SNN_TUNE_SUBBIT_MFMA 0 /* 0: layers the matrix-core kernel supports go to the LDS-gather kernel */
#define SNN_TUNE_MFMA_TILE   1 /* 10 * PB + CB, blocks of 32 pixels x 32 channels per wave: 42, 24, 22, 14, 12 */
#define SNN_TUNE_MFMA_KS     2 /* waves that share a tile's input channels: 1, 2, 4 */
#define SNN_TUNE_MFMA_STAGE  3 /* 0 / 1: packed rows staged in LDS wherever they fit */
#define SNN_TUNE_MFMA_QUAD   4 /* 0 / 1: four channels per matrix instruction wherever K <= 16 */
#define SNN_TUNE_STACK       5 /* 0: snn_subbit_conv2d_prepared_many runs one workgroup per tile group */
#define SNN_TUNE_BNN_REGS    6 /* 0: the 1-bit kernel without register-resident windows */
#define SNN_TUNE_DENSE_TILE  7 /* 0 .. 4: tile shape of the dense contraction */
#define SNN_TUNE_F32_WAVES   8 /* 4, 8, 16: waves per workgroup of the fp32-activation sub-bit kernel */
#define SNN_TUNE_COUNT       9
int snn_set_tuning(int knob, int value);
int snn_get_tuning(int knob); /* SNN_TUNE_AUTO for an unknown knob */

#ifdef __cplusplus
}
#endif
#endif /* SNN_H */

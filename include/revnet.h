/*
 * revnet.h -- C ABI of the MI355X (gfx950) reversible-residual-block library.
 *
 * The library runs the hot path of "The Reversible Residual Network:
 * Backpropagation Without Storing Activations" (Gomez, Ren, Urtasun, Grosse,
 * 2017): the forward pass of a reversible block and the backward pass that
 * reconstructs the block's inputs from its outputs instead of reading stored
 * activations, for single blocks and for stacks of blocks.  Further entry
 * points build whole networks around such stacks: the non-reversible
 * subsampling block between stages, the multi-stage body, the stem, and a
 * variant that keeps the residual stream in fixed point (exact reconstruction).
 *
 * Conventions common to every entry point
 * ---------------------------------------
 * Memory.   Every pointer inside rvn_tensor / rvn_func_params / rvn_func_grads
 *           and every `ws` pointer is a DEVICE pointer.  The descriptor,
 *           tensor and parameter structs themselves live in HOST memory and
 *           are read during the call only.  The caller owns all device
 *           buffers, including the workspace; the library allocates and frees
 *           nothing on the device and keeps no state between calls.
 * Stream.   All work is enqueued on `hip_stream` (a hipStream_t cast to
 *           void*; NULL = the default stream).  Nothing synchronises with the
 *           host; buffers must stay valid until the stream has drained.
 * Tensors.  Residual-stream tensors are fp32, logical shape [n, c, h, w],
 *           strides in ELEMENTS.  Supported memory layout: sw == 1,
 *           sh == w, sc >= h*w, sn >= (c-1)*sc + h*w (rows and planes
 *           contiguous; channel and image strides free).  This lets x1 and
 *           x2 be the two channel halves of one [N, C, H, W] buffer without a
 *           copy (Section 3.1: the units are partitioned by channels; x1 is
 *           channels [0, C/2), x2 is [C/2, C)).  Other strides give
 *           RVN_ERR_STRIDE.
 * Params.   conv_w[l] is dense fp32 [c_out][c_in][k][k]; bn_gamma[l],
 *           bn_beta[l] are fp32 [c_in] (the BN sits in front of conv l).
 *           Layer shapes follow from the descriptor:
 *             RVN_BASIC      : (c_half -> c_half, 3x3), (c_half -> c_half, 3x3)
 *             RVN_BOTTLENECK : (c_half -> width, 1x1), (width -> width, 3x3),
 *                              (width -> c_half, 1x1)
 *           (Section 2.2, the equations for a(x), c_k(x), Basic, Bottleneck).
 *           Unused slots are ignored.
 * Errors.   Every entry point returns RVN_OK (0) or a negative rvn_status.
 *           All argument checks happen before the first device call, so a
 *           rejected call has touched nothing.  revnet_last_error() returns a
 *           message for the calling thread's most recent failure.
 * Numerics. Batch normalisation always uses the statistics of the batch at
 *           hand (biased variance, eps inside the square root) and keeps no
 *           running averages; ReLU'(0) = 0; convolutions are stride 1
 *           (Section 3.1: reversible blocks must have stride 1), zero padded
 *           by (k-1)/2, without bias.  conv_dtype selects the precision of the
 *           convolution OPERANDS only (activations after BN+ReLU, filters,
 *           and the upstream gradient where it enters a convolution); sums,
 *           BN, the residual stream and all gradients are fp32.
 *           Every kernel is deterministic (no floating-point atomics): the
 *           same call on the same inputs gives the same bits.  With the
 *           floating-point stream the backward pass may form the batch
 *           statistics of a stream tensor in another summation order than the
 *           forward pass did (a full pass over the tensor against partial
 *           sums left by the convolution that produced it), so a recomputed
 *           G(y1) agrees with the forward one to fp32 rounding, not bit for
 *           bit; the reconstruction error is that plus the rounding of
 *           (x + g) - g (Section 3.2, "Numerical error").  The fixed-point
 *           entry points further down take every statistic of a stream tensor
 *           from one algorithm in both passes and reconstruct bit for bit.
 * Diagnostics. While the environment variable RVN_SEPARATE_LAUNCHES is "1" the
 *           backward pass gives the data gradient and the filter gradient of
 *           a layer a launch each instead of one shared launch (the default).
 *           It is read at every call; results are the same bits either way,
 *           the launch counts of the cost queries follow it.
 */
#ifndef REVNET_H
#define REVNET_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RVN_OK = 0,
    RVN_ERR_NULL = -1,        /* a required pointer is NULL                       */
    RVN_ERR_SHAPE = -2,       /* non-positive or inconsistent n/c/h/w/depth/width */
    RVN_ERR_STRIDE = -3,      /* memory layout outside the supported family       */
    RVN_ERR_DTYPE = -4,       /* unknown rvn_dtype / rvn_kind                     */
    RVN_ERR_WORKSPACE = -5,   /* ws is NULL, misaligned (256 B) or too small      */
    RVN_ERR_ALIAS = -6,       /* buffers overlap in a way the contract forbids    */
    RVN_ERR_UNSUPPORTED = -7, /* valid request this build cannot run              */
    RVN_ERR_HIP = -8          /* a HIP runtime call or kernel launch failed       */
} rvn_status;

typedef enum { RVN_F32 = 0, RVN_BF16 = 1 } rvn_dtype;
typedef enum { RVN_BASIC = 0, RVN_BOTTLENECK = 1 } rvn_kind;

/* fp32 device tensor, logical NCHW, strides in elements. */
typedef struct {
    void *ptr;
    int64_t n, c, h, w;
    int64_t sn, sc, sh, sw;
} rvn_tensor;

typedef struct {
    rvn_kind kind;
    int32_t c_half;       /* channels of x1 (= channels of x2)              */
    int32_t width;        /* bottleneck inner channels; ignored for BASIC   */
    float bn_eps;         /* > 0                                            */
    rvn_dtype conv_dtype; /* precision of convolution operands              */
} rvn_block_desc;

typedef struct {
    const float *conv_w[3];
    const float *bn_gamma[3];
    const float *bn_beta[3];
} rvn_func_params;

typedef struct {
    float *d_conv_w[3];
    float *d_bn_gamma[3];
    float *d_bn_beta[3];
} rvn_func_grads;

typedef struct { rvn_func_params F, G; } rvn_block_params;
typedef struct { rvn_func_grads F, G; } rvn_block_grads;

/* Work a call enqueues, counted by the same driver code that launches it
 * (the driver is run without touching the device). */
typedef struct {
    int64_t kernel_launches;
    int64_t conv_fwd_calls;   /* convolution forward evaluations            */
    int64_t conv_dgrad_calls; /* data-gradient evaluations                  */
    int64_t conv_wgrad_calls; /* filter-gradient evaluations                */
    double conv_flops;        /* 2 * multiply-adds of the three above       */
    double algorithmic_bytes; /* sum over launches of bytes each must move  */
} rvn_cost;

/*
 * Workspace sizes, in bytes, for blocks of this descriptor on [n, c_half, h, w]
 * halves.  fwd_bytes serves revnet_block_fwd / revnet_stack_fwd, bwd_bytes
 * serves revnet_block_bwd_reconstruct / revnet_stack_bwd.  Neither depends on
 * the depth of a stack: only one residual function's internals are alive at a
 * time (Section 3.2: activation storage independent of depth).  Either output
 * pointer may be NULL.
 */
int revnet_workspace_bytes(const rvn_block_desc *desc, int64_t n, int64_t h, int64_t w,
                           size_t *fwd_bytes, size_t *bwd_bytes);

/*
 * Reversible block, forward (Section 3.1, the forward coupling equations):
 *     y1 = x1 + F(x2)
 *     y2 = x2 + G(y1)
 * x1, x2: inputs [n, c_half, h, w] (read).  y1, y2: outputs, same shape
 * (written).  y1 may be the same tensor as x1 and y2 the same as x2 (same ptr
 * and strides: in-place update); any other overlap among the four, or with
 * the workspace, is RVN_ERR_ALIAS.  ws: >= fwd_bytes, 256-byte aligned.
 */
int revnet_block_fwd(const rvn_block_desc *desc,
                     const rvn_tensor *x1, const rvn_tensor *x2,
                     const rvn_block_params *params,
                     const rvn_tensor *y1, const rvn_tensor *y2,
                     void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Reversible block, backward without stored activations (Section 3.2,
 * Algorithm 1).  From the block's outputs (y1, y2) and their total
 * derivatives (dy1, dy2) alone it returns the block's inputs, their total
 * derivatives and the parameter derivatives.  Data flow: G is evaluated once
 * at y1, which gives x2 = y2 - G(y1) and, by ordinary backprop through the
 * activations of that evaluation, dwG and the derivative reaching y1's node,
 * dx1 = dy1 + (dG/dy1)^T dy2; F is then evaluated once at the recovered x2,
 * which gives x1 = y1 - F(x2), dwF and dx2 = dy2 + (dF/dx2)^T dx1.
 * (Section 5.1: back-propagating through the activations of the two
 * reconstruction evaluations gives the 4N total cost of Section 3.2.)  Only
 * one function's internals are alive at a time.
 * y1, y2, dy1, dy2: read.  x1, x2, dx1, dx2: written.  x_i may be the same
 * tensor as y_i and dx_i the same as dy_i (in place); any other overlap is
 * RVN_ERR_ALIAS.  grads: every pointer of the layers the descriptor uses must
 * be non-NULL; each is overwritten, or added to when accumulate_wgrads != 0
 * (weight sharing across blocks, Section 3.2 footnote on Algorithm 1).
 * ws: >= bwd_bytes, 256-byte aligned.
 */
int revnet_block_bwd_reconstruct(const rvn_block_desc *desc,
                                 const rvn_tensor *y1, const rvn_tensor *y2,
                                 const rvn_tensor *dy1, const rvn_tensor *dy2,
                                 const rvn_block_params *params,
                                 const rvn_tensor *x1, const rvn_tensor *x2,
                                 const rvn_tensor *dx1, const rvn_tensor *dx2,
                                 const rvn_block_grads *grads, int accumulate_wgrads,
                                 void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Stack of `depth` reversible blocks of one descriptor, forward (Section 3.2,
 * the paragraph on sequences of blocks): block k maps its input pair to its
 * output pair with params[k], k = 0 .. depth-1; only the top pair (y1, y2) is
 * produced, no per-block activation is kept.  params: host array [depth].
 * Aliasing as in revnet_block_fwd (block 0 reads x and writes y; later blocks
 * update y in place).
 */
int revnet_stack_fwd(const rvn_block_desc *desc, int32_t depth,
                     const rvn_tensor *x1, const rvn_tensor *x2,
                     const rvn_block_params *params,
                     const rvn_tensor *y1, const rvn_tensor *y2,
                     void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Stack backward (Section 3.2: Algorithm 1 applied repeatedly, given only the
 * top activations and their derivatives), k = depth-1 .. 0.  Writes the
 * reconstructed stack input (x1, x2), its derivatives (dx1, dx2) and the
 * parameter gradients of every block (grads: host array [depth]).  Block
 * depth-1 reads (y, dy) and writes (x, dx); lower blocks update (x, dx) in
 * place.  Aliasing as in revnet_block_bwd_reconstruct.  With
 * accumulate_wgrads != 0 two blocks may share gradient buffers.
 */
int revnet_stack_bwd(const rvn_block_desc *desc, int32_t depth,
                     const rvn_tensor *y1, const rvn_tensor *y2,
                     const rvn_tensor *dy1, const rvn_tensor *dy2,
                     const rvn_block_params *params,
                     const rvn_tensor *x1, const rvn_tensor *x2,
                     const rvn_tensor *dx1, const rvn_tensor *dx2,
                     const rvn_block_grads *grads, int accumulate_wgrads,
                     void *ws, size_t ws_bytes, void *hip_stream);

/*
 * revnet_stack_fwd for callers that cannot allocate device memory and hold no
 * workspace of their own: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, kernels and results as
 * revnet_stack_fwd, without `ws` / `ws_bytes`: the workspace is a fixed array
 * of RVN_STATIC_WS_BYTES inside the library's device image (one copy per GPU
 * that uses the library, held until the process ends).  The call allocates
 * and frees nothing, on the device or through any library.
 * Limit: shapes whose forward workspace (revnet_workspace_bytes: fwd_bytes)
 * exceeds RVN_STATIC_WS_BYTES are rejected with RVN_ERR_WORKSPACE before
 * anything is enqueued.
 * Sharing: every call on one GPU uses that GPU's one array, on whatever
 * stream.  Calls on the same stream are ordered and safe; calls whose work
 * can overlap on one GPU (different streams, different host threads without
 * stream ordering) race on the array and give undefined results.  The array
 * keeps the previous call's contents; the call itself clears what it needs
 * zeroed (with a kernel, so it can be captured).
 * The first call on a device looks up the array's address
 * (hipGetSymbolAddress); make that call outside stream capture.
 */
#define RVN_STATIC_WS_BYTES ((size_t)32 << 20)
int revnet_stack_fwd_static(const rvn_block_desc *desc, int32_t depth,
                            const rvn_tensor *x1, const rvn_tensor *x2,
                            const rvn_block_params *params,
                            const rvn_tensor *y1, const rvn_tensor *y2,
                            void *hip_stream);

/* ------------------------------------------------------------------------
 * Non-reversible subsampling block and multi-stage body.
 *
 * A reversible block has stride 1 (Section 3.1), so a network also holds
 * ordinary layers that change the resolution; their inputs are stored
 * (Section 3.2, last paragraph on storage).  The paper does not give their
 * form.  The one built here is a pre-activation residual block on the whole
 * tensor x [n, c_in, h, w] -> y [n, c_out, h/2, w/2] (h and w even):
 *     a0 = ReLU(BN_0(x))
 *     y  = Conv_1x1,stride 2(a0; shortcut_w) + R(x)
 * with R the Basic function c3(c3(x)) or the Bottleneck function c1(c3(c1(x)))
 * of Section 2.2, stride 2 on its (first) 3x3 convolution:
 *     basic:      (c_in -> c_out, 3x3, stride 2), (c_out -> c_out, 3x3)
 *     bottleneck: (c_in -> width, 1x1), (width -> width, 3x3, stride 2), (width -> c_out, 1x1)
 * BN_0 is the BN of R's first unit: the shortcut reads the same pre-activation.
 * ---------------------------------------------------------------------- */
typedef struct {
    rvn_kind kind;
    int32_t c_in, c_out;  /* channels of the whole input / output tensor */
    int32_t width;        /* bottleneck inner width; ignored for RVN_BASIC */
    float bn_eps;
    rvn_dtype conv_dtype;
} rvn_down_desc;

typedef struct {
    rvn_func_params R;       /* layers as listed above */
    const float *shortcut_w; /* [c_out][c_in], device */
} rvn_down_params;

typedef struct {
    rvn_func_grads R;
    float *d_shortcut_w; /* [c_out][c_in], device */
} rvn_down_grads;

/* Workspace bytes for an input of n x c_in x h x w.  Either pointer may be NULL. */
int revnet_down_workspace_bytes(const rvn_down_desc *desc, int64_t n, int64_t h, int64_t w,
                                size_t *fwd_bytes, size_t *bwd_bytes);

/*
 * y = shortcut + R(x) as defined above.  x [n, c_in, h, w] is read and must be
 * kept by the caller for revnet_down_bwd; y [n, c_out, h/2, w/2] is written.
 * Tensors as in revnet_block_fwd (sw = 1, sh = w, sc >= h*w); x, y and the
 * workspace must not overlap.  Errors as for the block entry points.
 */
int revnet_down_fwd(const rvn_down_desc *desc, const rvn_tensor *x, const rvn_down_params *params,
                    const rvn_tensor *y, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Ordinary backprop (Section 2.1) through the subsampling block from its
 * stored input: the internals are recomputed from x, then dx = (dy/dx)^T dy
 * and the parameter gradients are formed.  x, dy: read.  dx [n, c_in, h, w]:
 * written; it must not overlap x, dy or the workspace.  grads: every pointer
 * of the layers in use and d_shortcut_w non-NULL; overwritten, or added to
 * when accumulate_wgrads != 0.
 */
int revnet_down_bwd(const rvn_down_desc *desc, const rvn_tensor *x, const rvn_tensor *dy,
                    const rvn_down_params *params, const rvn_tensor *dx, const rvn_down_grads *grads,
                    int accumulate_wgrads, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Body: `stages` stacks of reversible blocks, stage s at half the resolution
 * of stage s-1, joined by subsampling blocks (down[s] maps the output of stage
 * s to the input of stage s+1).  Only the top activation of every stage is
 * kept -- it is the stored input of the subsampling block above it -- so the
 * activation memory does not depend on the stages' depths (Section 3.2).
 * The body starts at the output of the network's first layers (stem, pooling),
 * which are not part of it.
 */
#define RVN_MAX_STAGES 8
typedef struct {
    int32_t stages;
    rvn_block_desc stage[RVN_MAX_STAGES]; /* c_half = half the stage's channels */
    int32_t depth[RVN_MAX_STAGES];        /* reversible blocks per stage, >= 1 */
    rvn_down_desc down[RVN_MAX_STAGES];   /* [stages - 1]; down[s].c_in = 2*stage[s].c_half,
                                             down[s].c_out = 2*stage[s+1].c_half */
} rvn_body_desc;

/* Workspace bytes for a body whose first stage sees n x (2*stage[0].c_half) x h x w. */
int revnet_body_workspace_bytes(const rvn_body_desc *desc, int64_t n, int64_t h, int64_t w,
                                size_t *fwd_bytes, size_t *bwd_bytes);

/*
 * Body forward.  x [n, C_0, h, w]: read.  tops: host array [stages] of
 * tensors, tops[s] = [n, C_s, h >> s, w >> s], dense (sc = h_s*w_s,
 * sn = C_s*sc); all are written: tops[s] is the output of stage s and
 * tops[stages-1] the body's output.  Channels [0, C_s/2) of a stage's tensor
 * are x1, the others x2 (Section 3.1: the channels are partitioned).
 * stage_params: host array [stages] of host arrays [depth[s]]; down_params:
 * host array [stages-1].  x may be tops[0] itself (then stage 0 runs in
 * place); no other overlap.
 */
int revnet_body_fwd(const rvn_body_desc *desc, const rvn_tensor *x,
                    const rvn_block_params *const *stage_params, const rvn_down_params *down_params,
                    const rvn_tensor *tops, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Body backward from the stored tops alone.  tops: as left by revnet_body_fwd;
 * every stage is reconstructed in place by Algorithm 1, so on return tops[s]
 * holds the reconstructed input of stage s (tops[0]: the body's input).
 * dtops: host array [stages] of tensors shaped like tops; dtops[stages-1]
 * holds the derivative with respect to the body's output on entry; all are
 * overwritten, and on return dtops[s] is the derivative with respect to the
 * input of stage s (dtops[0]: with respect to the body's input).
 * stage_grads / down_grads: shaped like the parameters.
 */
int revnet_body_bwd(const rvn_body_desc *desc, const rvn_tensor *tops, const rvn_tensor *dtops,
                    const rvn_block_params *const *stage_params, const rvn_down_params *down_params,
                    const rvn_block_grads *const *stage_grads, const rvn_down_grads *down_grads,
                    int accumulate_wgrads, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * The body with a fixed-point residual stream (see revnet_stack_fwd_fixed
 * further down for the format): tops hold int32 codes of 2^-frac_bits, x and
 * dtops stay fp32.  x is encoded into tops[0]; a subsampling block reads its
 * stored input decoded to fp32, and its fp32 output is encoded (rounded to the
 * nearest code) into the next stage's tensor.  Every stage then reconstructs
 * bit for bit in revnet_body_bwd_fixed, so the whole backward pass runs at
 * exactly the forward activations.  x may be tops[0] itself (encoded in place).
 */
int revnet_body_fixed_workspace_bytes(const rvn_body_desc *desc, int64_t n, int64_t h, int64_t w,
                                      size_t *fwd_bytes, size_t *bwd_bytes);
int revnet_body_fwd_fixed(const rvn_body_desc *desc, int32_t frac_bits, const rvn_tensor *x,
                          const rvn_block_params *const *stage_params, const rvn_down_params *down_params,
                          const rvn_tensor *tops, void *ws, size_t ws_bytes, void *hip_stream);
int revnet_body_bwd_fixed(const rvn_body_desc *desc, int32_t frac_bits, const rvn_tensor *tops,
                          const rvn_tensor *dtops,
                          const rvn_block_params *const *stage_params, const rvn_down_params *down_params,
                          const rvn_block_grads *const *stage_grads, const rvn_down_grads *down_grads,
                          int accumulate_wgrads, void *ws, size_t ws_bytes, void *hip_stream);

/* ------------------------------------------------------------------------
 * Stem: the network's first layers, ahead of the body.  Non-reversible, so
 * their inputs are stored (Section 3.2).  The paper follows the residual
 * networks it cites for these layers; built here: a k x k convolution of the
 * image (k = 1, 3, 5 or 7, c_in * k * k <= 256, stride 1 or 2, zero padding (k-1)/2, no
 * bias, fp32), optionally followed by max-pooling over 3x3 windows with stride
 * 2 and padding 1.  img [n, c_in, h, w] -> conv_out [n, c_out, ho, wo],
 * ho = (h-1)/stride + 1; with pool != 0: y [n, c_out, (ho-1)/2 + 1, (wo-1)/2 + 1].
 * ---------------------------------------------------------------------- */
typedef struct {
    int32_t c_in, c_out, ks, stride;
    int32_t pool; /* 0: the convolution's output is the stem's output */
} rvn_stem_desc;

/* Workspace bytes revnet_stem_bwd needs for an image batch of n x c_in x h x w. */
int revnet_stem_workspace_bytes(const rvn_stem_desc *desc, int64_t n, int64_t h, int64_t w, size_t *bwd_bytes);

/*
 * img: read.  w: filter [c_out][c_in][ks][ks], device.  pool == 0: y receives
 * the convolution and conv_out must be NULL.  pool != 0: conv_out receives the
 * convolution (the caller keeps it for revnet_stem_bwd: it is the stored input
 * of the pooling layer) and y the pooled result.  No overlaps.
 */
int revnet_stem_fwd(const rvn_stem_desc *desc, const rvn_tensor *img, const float *w,
                    const rvn_tensor *conv_out, const rvn_tensor *y, void *hip_stream);

/*
 * d_w (+)= derivative with respect to the filter, from the stored img (and
 * conv_out when pool != 0, else NULL) and dy, the derivative with respect to
 * the stem's output.  A pooling window passes its derivative to its first
 * maximal element in row-major order.  The image receives no derivative.
 */
int revnet_stem_bwd(const rvn_stem_desc *desc, const rvn_tensor *img, const rvn_tensor *conv_out,
                    const rvn_tensor *dy, float *d_w, int accumulate_wgrads,
                    void *ws, size_t ws_bytes, void *hip_stream);

/* ------------------------------------------------------------------------
 * Fixed-point residual stream (Section 3.2, "Numerical error": with the x's
 * and y's in fixed point and F, G in ordinary floating point the
 * reconstruction is exact, at little extra cost).
 *
 * Stream tensors (x1, x2, y1, y2) hold int32 codes q standing for
 * q * 2^-frac_bits, 1 <= frac_bits <= 30, in the same rvn_tensor layout
 * (strides in 4-byte elements).  A function reads float(q) * 2^-frac_bits; its
 * fp32 value f enters the stream as an integer sum,
 *     y1 = x1 + rint(F(x2) * 2^frac_bits),   y2 = x2 + rint(G(y1) * 2^frac_bits),
 * and the backward pass subtracts the same integers again, so x1, x2 come back
 * bit for bit, at any depth, and the functions are back-propagated at exactly
 * the activations of the forward pass.  Derivatives and parameters stay fp32.
 * Codes wrap around on overflow (the caller chooses frac_bits so that the
 * stream fits: |value| < 2^(31 - frac_bits)); the conversion of one function
 * value saturates.  Everything else as for revnet_stack_fwd / revnet_stack_bwd,
 * with the workspace size from revnet_fixed_workspace_bytes.
 * ---------------------------------------------------------------------- */
int revnet_fixed_workspace_bytes(const rvn_block_desc *desc, int64_t n, int64_t h, int64_t w,
                                 size_t *fwd_bytes, size_t *bwd_bytes);

/* dst (int32 codes) = rint(src * 2^frac_bits); src fp32.  dst may be src itself. */
int revnet_fixed_from_float(const rvn_tensor *src, int32_t frac_bits, const rvn_tensor *dst, void *hip_stream);

/* dst (fp32, dense: sc = h*w, sn = c*h*w) = src (int32 codes) * 2^-frac_bits.  No overlap. */
int revnet_fixed_to_float(const rvn_tensor *src, int32_t frac_bits, const rvn_tensor *dst, void *hip_stream);

int revnet_stack_fwd_fixed(const rvn_block_desc *desc, int32_t depth, int32_t frac_bits,
                           const rvn_tensor *x1, const rvn_tensor *x2,
                           const rvn_block_params *params,
                           const rvn_tensor *y1, const rvn_tensor *y2,
                           void *ws, size_t ws_bytes, void *hip_stream);

int revnet_stack_bwd_fixed(const rvn_block_desc *desc, int32_t depth, int32_t frac_bits,
                           const rvn_tensor *y1, const rvn_tensor *y2,
                           const rvn_tensor *dy1, const rvn_tensor *dy2,
                           const rvn_block_params *params,
                           const rvn_tensor *x1, const rvn_tensor *x2,
                           const rvn_tensor *dx1, const rvn_tensor *dx2,
                           const rvn_block_grads *grads, int accumulate_wgrads,
                           void *ws, size_t ws_bytes, void *hip_stream);

/*
 * What revnet_stack_fwd (fwd) and revnet_stack_bwd (bwd) would enqueue for
 * this descriptor, depth and half-tensor shape, without touching the device.
 * Lets a caller check the paper's operation count (Section 3.2,
 * "Computational overhead": forward N, reversible backward 3N) and gives the
 * flop and byte totals for roofline reports.  Either output may be NULL.
 */
int revnet_stack_cost(const rvn_block_desc *desc, int32_t depth,
                      int64_t n, int64_t h, int64_t w,
                      rvn_cost *fwd, rvn_cost *bwd);

/*
 * Per-kernel timing for roofline reports (not part of the paper's method).
 * Between revnet_profile_begin() and revnet_profile_end() every kernel the
 * library launches is bracketed by HIP events on the stream it is launched
 * on.  revnet_profile_end() waits for those events and returns, per kernel
 * family that ran, the number of launches, their summed duration, and the
 * summed algorithmic bytes and flops (the same figures revnet_stack_cost
 * counts).  stats: host array of max_stats entries; *n_stats receives the
 * number of families that ran.  `name` points to static storage.  Process
 * wide; events cost a few microseconds per launch, so time throughput in a
 * separate pass.
 */
typedef struct {
    const char *name;
    int64_t launches;
    double total_ms;
    double algorithmic_bytes;
    double flops;
} rvn_kernel_stat;

int revnet_profile_begin(void);
int revnet_profile_end(rvn_kernel_stat *stats, int32_t max_stats, int32_t *n_stats);

/* Message for the calling thread's most recent failing call ("" if none).
 * The storage is thread local and valid until that thread's next call. */
const char *revnet_last_error(void);

/* ABI version: major * 1000 + minor. */
int revnet_version(void);

#ifdef __cplusplus
}
#endif
#endif /* REVNET_H */

/*
 * libsol_mi355 -- C ABI of the fused CNN layer-chain engine for AMD MI355X (gfx950).
 *
 * The library executes what the paper's optimizing backend accelerates: the
 * forward (and, for training, backward) pass of a CNN layer chain, with the
 * convolution / linear layers run as dense contractions on the matrix cores
 * and their memory-bound neighbours (batch-norm, bias, ReLU, residual add,
 * pooling) fused into them (paper Sec. III-A: layer fusion that keeps data in
 * registers and caches; conv/linear as the work-intensive layers).
 *
 * Boundary conventions, after the paper's runtime (Sec. III-B: kernels read and
 * write the framework's tensors in place, the framework stays the only
 * allocator; Sec. III-A: optimise once, call many times):
 *
 *  - every data pointer is a DEVICE pointer owned by the caller; the library
 *    allocates no device memory and keeps no reference after a call returns,
 *    except for the buffers explicitly bound to a sol_network;
 *  - every call only enqueues work on `hip_stream` (a hipStream_t passed as
 *    void*, NULL = default stream) and returns without synchronising;
 *  - activations are dense NHWC: element (n,c,h,w) lives at ((n*H+h)*W+w)*C+c;
 *    documentation and pooling argmax use logical (n,c,h,w) indices;
 *  - arguments are validated before anything is launched; on error nothing was
 *    enqueued, a status code is returned and sol_last_error() holds the text;
 *  - device buffers must be 16-byte aligned; tensors hold fewer than 2^31 elements.
 */
#ifndef SOL_MI355_H
#define SOL_MI355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SOL_OK = 0,
    SOL_ERR_NULL = 1,        /* a required pointer is NULL */
    SOL_ERR_SHAPE = 2,       /* inconsistent or non-positive sizes */
    SOL_ERR_DTYPE = 3,       /* unknown element type */
    SOL_ERR_ALIGN = 4,       /* pointer not 16-byte aligned */
    SOL_ERR_WORKSPACE = 5,   /* a caller-provided buffer is too small */
    SOL_ERR_UNSUPPORTED = 6, /* valid request outside what the kernels implement */
    SOL_ERR_HIP = 7          /* the HIP runtime reported an error */
} sol_status;

typedef enum { SOL_F32 = 0, SOL_BF16 = 1 } sol_dtype;  /* bf16 = bf16 storage, fp32 accumulate */
typedef enum { SOL_ACT_NONE = 0, SOL_ACT_RELU = 1 } sol_act;
typedef enum { SOL_POOL_NONE = 0, SOL_POOL_MAX = 1, SOL_POOL_AVG = 2 } sol_pool_kind;
typedef enum { SOL_LAYER_CONV = 0, SOL_LAYER_POOL = 1, SOL_LAYER_GAP = 2, SOL_LAYER_LINEAR = 3, SOL_LAYER_DWCONV = 4,
               SOL_LAYER_CONCAT = 5 } sol_layer_kind;

/* sliding-window pooling; floor-mode output size; count_pad selects the average-pool divisor
 * (window area vs. number of in-range elements), the switch of the paper's pooling description
 * (Sec. IV, AveragePooling listing: K.area(isCountPadding)) */
typedef struct { int kind, kh, kw, sh, sw, ph, pw, count_pad; } sol_pool_desc;
typedef struct { int n, h, w, c; int dtype; } sol_tensor_desc;       /* dense NHWC */
typedef struct { int cout, cin, kh, kw, sh, sw, ph, pw; } sol_conv_desc;

/* one entry of a layer list; src / res are absolute indices of the producing layer
 * (src = -1: previous layer, or the network input for layer 0; res = -1: no residual).
 * CONCAT: output channels = [channels of layer src | channels of layer res], two different earlier layers of
 * equal n, h, w (the join of parallel branches in the SqueezeNet / DenseNet-shaped networks of the paper's
 * evaluation, Sec. VI); inference networks only; no parameters. */
typedef struct {
    int kind;               /* sol_layer_kind */
    sol_conv_desc conv;     /* CONV, DWCONV: cin is inferred and may be 0 (DWCONV: cout too) */
    int has_bn;             /* CONV, DWCONV: batch-norm follows the convolution */
    int act;                /* CONV, DWCONV, LINEAR: sol_act */
    sol_pool_desc pool;     /* CONV: pool fused behind the activation (kind NONE = none); POOL: the pool */
    int out_features;       /* LINEAR */
    int src, res;
    int pre_bn;             /* CONV: a batch-norm + ReLU of the layer's INPUT runs in front of the convolution (pre-activation
                               order, as in the DenseNet-shaped networks of the paper's evaluation, Sec. VI); its parameters
                               come through sol_network_set_pre_bn; the zero padding applies to the activated tensor;
                               inference networks only */
} sol_layer;

typedef struct sol_network sol_network;

const char *sol_last_error(void);   /* thread-local text of the last failure on this thread */
const char *sol_version(void);

/* ---- parameter preparation (run once per model: the paper's optimise step, Sec. III-A) -------- */

/* Bytes of the packed form of a convolution weight: [cout][kh][kw][cin] in `dt`, each output
 * channel's kh*kw*cin run zero-padded to a multiple of 64 (bf16) / 32 (fp32) elements. */
size_t sol_packed_weight_bytes(const sol_conv_desc *cd, sol_dtype dt);

/* w_oihw: device fp32 [cout][cin][kh][kw]  ->  w_packed (device, sol_packed_weight_bytes).
 * bf16 packing rounds to nearest even. */
sol_status sol_pack_conv_weights(const sol_conv_desc *cd, sol_dtype dt, const float *w_oihw,
                                 void *w_packed, void *hip_stream);

/* Inverse of the packing, widened to fp32 OIHW (used after an SGD step and by tests). */
sol_status sol_unpack_conv_weights(const sol_conv_desc *cd, sol_dtype dt, const void *w_packed,
                                   float *w_oihw, void *hip_stream);

/* Fold inference batch-norm and the convolution bias into one per-channel affine map (fp32, device):
 *   scale = gamma / sqrt(var + eps),  shift = beta - mean*scale + bias*scale.
 * gamma/beta/mean/var may all be NULL (no BN: scale = 1, shift = bias); bias may be NULL (0). */
sol_status sol_fold_bn(int c, const float *gamma, const float *beta, const float *mean,
                       const float *var, const float *bias, float eps, float *scale, float *shift,
                       void *hip_stream);

/* ---- single fused layers ----------------------------------------------------------------------- */

/* y = pool( act( scale[k] * conv(x, w)[.,k] + shift[k] + residual ) )
 * (the fused block of the problem statement: conv, folded BN, residual, ReLU, optional pool).
 *   xd, x      input NHWC, dtype xd->dtype (SOL_F32 or SOL_BF16); cd->cin must equal xd->c
 *   w_packed   from sol_pack_conv_weights with the same cd and dtype
 *   scale,shift device fp32 [cout]; NULL = 1 / 0
 *   residual   NULL or NHWC [n][Ho][Wo][cout] of the same dtype (conv-output shape, before pooling)
 *   pool       NULL or kind NONE = no pool.  Fused: max or avg, 2x2 window, stride 2, no padding
 *              (floor mode: an odd last row/column is dropped), behind any convolution; or a 3x3
 *              stride-2 pad-1 max pool behind a bf16 7x7 stride-2 convolution of a 3-channel input
 *              with 64 filters, ReLU and no residual (the ResNet-shaped stem pair, run depth-first
 *              in one kernel: y is [n][Hy][Wy][64] with Hy = sol_out_size(Ho, 3, 2, 1); pool_argmax
 *              and prepool must be NULL).  Any other pool -> SOL_ERR_UNSUPPORTED (run sol_pool on
 *              the result instead).
 *   y          NHWC [n][Hy][Wy][cout], same dtype as x
 *   pool_argmax NULL, or int32 NHWC like y (max pool only): logical index ih*Wo+iw of the winning
 *              element inside its (n,k) conv-output plane; among equal values the first in row-major
 *              window order wins.
 *   prepool    NULL, or a buffer of the conv-output shape that receives act(...) before pooling
 *              (same dtype as y; lets a caller check pooled values and indices on identical inputs).
 * Accumulation is fp32 for both dtypes; fp32 inputs use true fp32 multiplies. */
sol_status sol_conv2d_fused(const sol_tensor_desc *xd, const void *x, const sol_conv_desc *cd,
                            const void *w_packed, const float *scale, const float *shift,
                            const void *residual, int act, const sol_pool_desc *pool, void *y,
                            int32_t *pool_argmax, void *prepool, void *hip_stream);

/* The fused block with a batch-norm + ReLU on the INPUT side as well (pre-activation order; the paper names the
 * DenseNet-shaped networks, built from such layers on concatenated features, among its largest gains, Sec. VI):
 *   y = pool( act( scale[k] * conv( relu(pre_scale[c] * x + pre_shift[c]), w )[.,k] + shift[k] + residual ) )
 * Taps in the padding contribute 0 (the padding surrounds the activated tensor).  For bf16 the activated input is
 * rounded to bf16 before it is multiplied.  Arguments as sol_conv2d_fused, plus
 *   ldx        elements between consecutive input pixels: 0 or xd->c for a dense tensor, more when x is a channel
 *              prefix of a wider NHWC tensor (ldx * element size a multiple of 16)
 *   pre_scale, pre_shift  device fp32 [xd->c] (sol_fold_bn of the input-side BN), or both NULL: no input-side map
 * Runs on the register-staged kernel, which transforms the data on its way to on-chip memory; the 2x2 pools can be
 * fused as usual, winners and the pre-pool tensor are not offered. */
sol_status sol_conv2d_preact_fused(const sol_tensor_desc *xd, const void *x, int ldx, const float *pre_scale, const float *pre_shift,
                                   const sol_conv_desc *cd, const void *w_packed, const float *scale, const float *shift,
                                   const void *residual, int act, const sol_pool_desc *pool, void *y, void *hip_stream);

/* A whole residual bottleneck as one depth-first kernel (the paper's layer-chain fusion, Sec. III-A: a chain of layers
 * is run over a block of data while it sits in registers and on-chip memory, here across three contractions):
 *   t1 = relu(scale1 * conv1x1(x,  w1) + shift1)           c   -> mid channels
 *   t2 = relu(scale2 * conv3x3(t1, w2) + shift2)           mid -> mid, stride 1, pad 1
 *   y  = relu(scale3 * conv1x1(t2, w3) + shift3 + x)       mid -> c,   identity shortcut
 * t1 and t2 never reach device memory; they are rounded to the storage type where the layer-by-layer path stores them.
 *   xd, x       block input NHWC, SOL_BF16
 *   mid         64 or 128; xd->c a multiple of 128; xd->w at most 126 (mid 64) / 79 (mid 128) columns; anything
 *               else -> SOL_ERR_UNSUPPORTED (run the three layers through sol_conv2d_fused)
 *   w1_packed   sol_pack_conv_weights of cd = {mid, c, 1,1, 1,1, 0,0};  w2_packed: {mid, mid, 3,3, 1,1, 1,1};
 *               w3_packed: {c, mid, 1,1, 1,1, 0,0}
 *   scale*, shift*  device fp32 per output channel of each convolution (sol_fold_bn), all required
 *   y           NHWC like x, written by the call; must not alias x */
sol_status sol_bottleneck_fused(const sol_tensor_desc *xd, const void *x, int mid, const void *w1_packed, const float *scale1,
                                const float *shift1, const void *w2_packed, const float *scale2, const float *shift2,
                                const void *w3_packed, const float *scale3, const float *shift3, void *y, void *hip_stream);

/* The last 1x1 convolution of one bottleneck and the first 1x1 convolution of the next as one depth-first kernel (the
 * paper's layer-chain fusion, Sec. III-A, across the border of two blocks):
 *   y = relu(scale3 * conv1x1(t, w3) + shift3 + shortcut)      c  -> c4 channels   (stored: later layers read it)
 *   z = relu(scale1 * conv1x1(y, w1) + shift1)                 c4 -> cz channels
 * z is contracted from y while y sits in on-chip memory, rounded to bf16 as stored; y is written once and not read back.
 *   td, t       input of the first convolution, NHWC, SOL_BF16, td->c = 256
 *   c4          a multiple of 128, at most 1024;  cz = 256 or 512; anything else -> SOL_ERR_UNSUPPORTED (run the two
 *               layers through sol_conv2d_fused)
 *   w3_packed   sol_pack_conv_weights of cd = {c4, 256, 1,1, 1,1, 0,0};  w1_packed: {cz, c4, 1,1, 1,1, 0,0}
 *   scale*, shift*  device fp32 per output channel of each convolution (sol_fold_bn), all required
 *   shortcut    NHWC [n][h][w][c4], added before the first ReLU, required
 *   y, z        NHWC [n][h][w][c4] / [n][h][w][cz], written by the call; must not alias the inputs or each other */
sol_status sol_expand_reduce_fused(const sol_tensor_desc *td, const void *t, int c4, const void *w3_packed, const float *scale3,
                                   const float *shift3, const void *shortcut, void *y, int cz, const void *w1_packed,
                                   const float *scale1, const float *shift1, void *z, void *hip_stream);

/* Depthwise convolution: a grouped convolution with one group -- one kh x kw filter -- per channel, which the
 * paper assigns to the fusion engine as a pooling layer with learned window weights (Sec. III-A) instead of
 * to the contraction path:
 *   y[n,p,q,c] = act( scale[c] * sum_{r,s} x[n, p*sh+r-ph, q*sw+s-pw, c] * w[c,r,s] + shift[c] + residual[n,p,q,c] )
 * (taps outside the image contribute 0).
 *   sol_packed_dw_weight_bytes   size of the packed weights: [kh*kw][c] in `dt`, rounded up to 16 bytes
 *   sol_pack_dwconv_weights      w_c1hw: device fp32 [c][1][kh][kw] -> w_packed (device); bf16 rounds to nearest even
 *   sol_dwconv2d_fused           xd, x: input NHWC; cd->cin and cd->cout must both equal xd->c; scale, shift: device
 *                                fp32 [c] or NULL (1 / 0); residual: NULL or NHWC of the output shape and dtype;
 *                                y: NHWC [n][Ho][Wo][c], same dtype as x, written by the call; no pool is fused.
 * fp32 accumulation in row-major tap order for both dtypes.  All buffers are the caller's; errors as elsewhere
 * (status code + sol_last_error), nothing is launched on an error. */
size_t sol_packed_dw_weight_bytes(int c, int kh, int kw, sol_dtype dt);
sol_status sol_pack_dwconv_weights(int c, int kh, int kw, sol_dtype dt, const float *w_c1hw, void *w_packed,
                                   void *hip_stream);
sol_status sol_dwconv2d_fused(const sol_tensor_desc *xd, const void *x, const sol_conv_desc *cd,
                              const void *w_packed, const float *scale, const float *shift,
                              const void *residual, int act, void *y, void *hip_stream);

/* y[m][o] = act( bias[o] + sum_i x[m][i] * w[o][i] ).  x [m][in_f], y [m][out_f] in `dt`;
 * w: [out_f][in_f] packed as a 1x1 convolution weight (sol_pack_conv_weights with
 * cd = {out_f, in_f, 1,1,1,1,0,0}); bias device fp32 [out_f] or NULL. */
sol_status sol_linear(int m, int in_f, int out_f, sol_dtype dt, const void *x, const void *w_packed,
                      const float *bias, int act, void *y, void *hip_stream);

/* Stand-alone pooling over NHWC x (max with optional int32 argmax as above, or average).
 * Padding acts as -inf for max and as 0 for average.  Requires pad < kernel. */
sol_status sol_pool(const sol_tensor_desc *xd, const void *x, const sol_pool_desc *pd, void *y,
                    int32_t *argmax, void *hip_stream);

/* Global average pool: y[n][c] = mean over h,w of x[n][h][w][c]; y has x's dtype. */
sol_status sol_global_avgpool(const sol_tensor_desc *xd, const void *x, void *y, void *hip_stream);

/* Output extent of a sliding window, floor mode: (in + 2*pad - k) / stride + 1. */
int sol_out_size(int in, int k, int stride, int pad);

/* ---- whole networks: plan once, run many -------------------------------------------------------- */

/* Validates the layer list against `input`, infers every shape, chooses per-layer kernels/tiles and
 * lays out the parameter and activation buffers.  Host-only; allocates no device memory.
 * flags: SOL_NET_KEEP_ACTIVATIONS keeps every layer's output alive in the workspace (otherwise a
 * buffer is reused once its last consumer has run); SOL_NET_TRAINING implies it. */
enum { SOL_NET_TRAINING = 1, SOL_NET_KEEP_ACTIVATIONS = 2 };
sol_status sol_network_create(const sol_layer *layers, int n_layers, const sol_tensor_desc *input,
                              int flags, sol_network **out);
void sol_network_destroy(sol_network *net);

size_t sol_network_param_bytes(const sol_network *net);      /* packed weights + folded scale/shift */
size_t sol_network_workspace_bytes(const sol_network *net);  /* activations between layers */
int sol_network_num_layers(const sol_network *net);
/* shape of a layer's output (layer = -1: the network output) */
sol_status sol_network_output_desc(const sol_network *net, int layer, sol_tensor_desc *out);

/* Hands the network a caller-owned device buffer of at least sol_network_param_bytes() that must
 * stay valid while the network is used. */
sol_status sol_network_bind_params(sol_network *net, void *param_buf, size_t bytes);

/* Packs one layer's parameters (device fp32, framework layout: conv w [cout][cin][kh][kw], linear
 * w [out][in]) into the bound buffer and folds BN (gamma..var NULL when the layer has no BN). */
sol_status sol_network_set_params(sol_network *net, int layer, const float *w, const float *gamma,
                                  const float *beta, const float *mean, const float *var,
                                  const float *bias, float eps, void *hip_stream);

/* Folds the input-side batch-norm of a CONV layer created with pre_bn (device fp32 [cin] each) into the bound buffer. */
sol_status sol_network_set_pre_bn(sol_network *net, int layer, const float *gamma, const float *beta, const float *mean,
                                  const float *var, float eps, void *hip_stream);

/* Runs the layer list: one launch per fused layer on the stream, activations ping-ponged inside
 * `workspace`.  x: network input (NHWC), y: output of the last layer. */
sol_status sol_network_forward(sol_network *net, const void *x, void *y, void *workspace,
                               size_t workspace_bytes, void *hip_stream);

/* For callers that cannot allocate device memory or hold a workspace of their own (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): sol_network_forward with the activations between the layers
 * kept in a static device array of the library, SOL_STATIC_WORKSPACE_BYTES per GPU, resident from the library's load
 * until the process ends.  The call allocates nothing (no hipMalloc / hipFree, no allocating library routine).
 *   net     an inference network (SOL_ERR_UNSUPPORTED for SOL_NET_TRAINING) whose sol_network_workspace_bytes() is at
 *           most SOL_STATIC_WORKSPACE_BYTES (else SOL_ERR_WORKSPACE, nothing launched)
 *   x, y    device pointers as for sol_network_forward (caller-owned input and output of the last layer)
 * Runs on the current device (the stream must belong to it).  Results are those of sol_network_forward bit for bit.
 * Every call on one GPU uses the same array, which keeps the previous call's contents; every buffer of a pass is
 * written before it is read, so nothing needs clearing, but two calls whose execution overlaps on one GPU (different
 * streams, or different threads) race on it: serialise them.  Kept activations (sol_network_layer_output) are not
 * reachable through this call. */
#define SOL_STATIC_WORKSPACE_BYTES (32u << 20)
sol_status sol_network_forward_static(sol_network *net, const void *x, void *y, void *hip_stream);

/* Debugging / sweeping aid for tests and tuning scripts (not a part of the layer semantics): forces the convolution
 * kernel / tile id used by later sol_conv2d_fused, sol_linear and sol_network_* calls of the CALLING THREAD
 * (0 = the library's own choice).  An id that does not fit a layer makes that call fail with SOL_ERR_UNSUPPORTED. */
void sol_debug_set_conv_tile(int tile);

/* Measured ceilings for the roofline report (benchmark aid; no layer arithmetic).
 *   sol_debug_probe_copy   a plain device-to-device copy of `bytes` (multiple of 16; 16-byte aligned, non-overlapping
 *                          device buffers) by a simple kernel: what HBM delivers, 2 * bytes of traffic per call;
 *   sol_debug_probe_mfma   `workgroups` workgroups of eight waves, each wave `iters` rounds of four independent
 *                          32x32x16 bf16 matrix instructions on register operands; *flop (host) receives the
 *                          floating-point operations of the launch; sink: device float the kernel may write. */
sol_status sol_debug_probe_copy(void *dst, const void *src, size_t bytes, void *hip_stream);
sol_status sol_debug_probe_mfma(int iters, int workgroups, float *sink, double *flop, void *hip_stream);

/* Plan-time micro auto-tune (the paper's optimizer picks per-layer implementations by heuristics or a very short
 * auto-tuning run when the model is optimized, Sec. III-A): times every kernel / tile shape that fits each
 * convolution layer, `reps` launches each on the caller's buffers, and keeps the fastest per layer for all later
 * sol_network_forward / sol_network_graph_create calls (the shape heuristic's choice stays unless a candidate is
 * more than 3 % faster).  Runs whole passes over x / workspace / y (their contents are overwritten with valid
 * activations), synchronises with the stream, allocates nothing on the device.  Every candidate computes the same
 * layer within the library's tolerance; the accumulation order, hence the last bits, may differ between candidates.
 * Training networks (SOL_NET_TRAINING): every convolution layer gets one choice for its forward convolution and
 * one for its data-gradient convolution, used by later sol_network_forward / sol_network_backward calls; the timed
 * launches overwrite activations and gradient buffers, so run a forward pass before the next backward.
 * sol_network_layer_tile reports the id chosen for the forward convolution (0 = heuristic). */
sol_status sol_network_autotune(sol_network *net, const void *x, void *y, void *workspace,
                                size_t workspace_bytes, int reps, void *hip_stream);
sol_status sol_network_layer_tile(const sol_network *net, int layer, int *tile);
/* Restores a choice that sol_network_autotune made earlier (same network, same machine): `tile` as reported by
 * sol_network_layer_tile, 0 = shape heuristic.  An id that does not fit the layer makes the next forward fail with
 * SOL_ERR_UNSUPPORTED before anything is launched for that layer. */
sol_status sol_network_set_layer_tile(sol_network *net, int layer, int tile);

/* Whole bottlenecks in one launch.  When a network keeps no activations (flags 0), bf16: a 1x1 convolution + ReLU, a
 * 3x3 stride-1 pad-1 convolution + ReLU and a 1x1 convolution + ReLU whose residual is the first one's input, each
 * intermediate read by the next layer only, with shapes sol_bottleneck_fused accepts, can run as that one depth-first
 * kernel; the plan decides by a shape heuristic, sol_network_autotune by timing both ways.  sol_network_layer_fused_into
 * reports the last convolution's index for the first two while the block runs fused.  sol_network_set_layer_block
 * restores / forces the choice for the block that ends in convolution `layer` (fused != 0: one launch;
 * SOL_ERR_UNSUPPORTED if `layer` ends no such block). */
sol_status sol_network_set_layer_block(sol_network *net, int layer, int fused);
/* *state = -1: `layer` ends no such block; 0: the block runs layer by layer; 1: as one launch */
sol_status sol_network_layer_block(const sol_network *net, int layer, int *state);

/* Expand -> reduce pairs in one launch.  When a network keeps no activations (flags 0), bf16: the last 1x1 convolution of
 * a bottleneck (+ shortcut, ReLU) followed directly by a 1x1 convolution + ReLU that reads only its output, with shapes
 * sol_expand_reduce_fused accepts, can run as that one kernel; both outputs are stored.  The plan decides by a shape
 * heuristic, sol_network_autotune by timing both ways.  sol_network_layer_fused_into reports the first layer's index
 * for the second while the pair runs fused.  *state = -1: `layer` starts no such pair; 0: the two run layer by layer;
 * 1: as one launch.  sol_network_set_layer_xr restores / forces the choice (SOL_ERR_UNSUPPORTED if `layer` starts no pair). */
sol_status sol_network_layer_xr(const sol_network *net, int layer, int *state);
sol_status sol_network_set_layer_xr(sol_network *net, int layer, int fused);

/* One forward pass recorded as a HIP graph (launch-bound inner loops: the about forty launches of a ResNet-50-shaped
 * pass replay as one submission).  sol_network_graph_create runs the pass once eagerly, then records the same
 * launches with the given pointers baked in: x, y, workspace, the bound parameter buffer and the network must
 * stay alive and unmoved while the graph is used (their CONTENTS may change between launches).  `hip_stream`
 * must be a real stream (not NULL, which cannot be captured); inference networks only.
 * sol_graph_launch enqueues one replay; launches on one stream run in order.  Records no memset nodes. */
typedef struct sol_graph sol_graph;
sol_status sol_network_graph_create(sol_network *net, const void *x, void *y, void *workspace,
                                    size_t workspace_bytes, void *hip_stream, sol_graph **out);
sol_status sol_graph_launch(sol_graph *graph, void *hip_stream);
void sol_graph_destroy(sol_graph *graph);

/* Fused layer pairs (the paper's layer-chain fusion, Sec. III-A and IV), when a network keeps no activations
 * (flags 0), bf16:
 *   - a 7x7 stride-2 convolution of a 3-channel input with 64 filters, ReLU and no residual whose only consumer is
 *     a 3x3 stride-2 pad-1 max-pool LAYER runs in one kernel with that pool; the convolution's output is never stored;
 *   - an unpadded 1x1 convolution (any stride) over a multiple of 64 channels without activation (a projection
 *     shortcut) whose only reader is the residual input of a later unpadded 1x1 stride-1 convolution over a multiple
 *     of 64 channels runs inside that convolution's launch; its output is never stored, and never rounded to the storage type either (the result differs from
 *     the two-launch result by at most one rounding of the shortcut term).
 * *into = index of the layer whose launch produces `layer`'s output: `layer` itself, the layer in front for such a
 * pool layer, the later convolution for such a shortcut, the last convolution of a bottleneck that runs as one launch
 * (see sol_network_set_layer_block) for its first two, the first layer of an expand -> reduce pair (see
 * sol_network_set_layer_xr) for its second (sol_network_run_layer on a fused layer launches nothing). */
sol_status sol_network_layer_fused_into(const sol_network *net, int layer, int *into);

/* Concatenation in place: when a network keeps no activations, a convolution (no fused pool, channel count a
 * multiple of 8) whose output is read by one CONCAT layer only writes its channels straight into that layer's
 * buffer, provided its slice starts on a multiple of 8 channels and the joined count is one too; the other
 * inputs are copied into place when the CONCAT layer runs.  A chain of CONCAT layers each of which extends the one
 * before it by new channels (a dense block: src = the previous CONCAT) shares ONE buffer of the final width when the
 * intermediate joins are read only by 1x1 convolutions, which then read a channel prefix of that buffer: the
 * features of a dense block are written once and never copied.  *parts = how many of the two inputs of CONCAT layer
 * `layer` are in place (2: the layer launches nothing).  SOL_ERR_SHAPE if `layer` is not a CONCAT. */
sol_status sol_network_concat_in_place(const sol_network *net, int layer, int *parts);

/* Runs one layer only, on whatever its producers left in the workspace (profiling aid: lets a caller
 * bracket a single layer with events).  Same arguments as sol_network_forward. */
sol_status sol_network_run_layer(sol_network *net, int layer, const void *x, void *y, void *workspace,
                                 size_t workspace_bytes, void *hip_stream);

/* Device address (inside the workspace passed to the last forward) of a layer's output; only
 * meaningful after a forward of a network created with SOL_NET_KEEP_ACTIVATIONS. */
sol_status sol_network_layer_output(const sol_network *net, int layer, void *workspace, void **ptr);

/* ---- training step (networks created with SOL_NET_TRAINING) ----------------------------------------
 * The layer-wise training semantics are those of the framework the paper extends (Sec. V: the
 * middleware inherits the framework's training loop; Sec. III: the forward layers above), with BN
 * using batch statistics.  On such a network:
 *   - fused pools are rejected at creation (the pool is a layer of its own), the last layer must produce
 *     [n,1,1,classes] logits, and sol_network_set_params ignores mean/var (NULL allowed) and keeps fp32
 *     master copies of w, gamma, beta, bias next to the packed weights, with zeroed velocities;
 *   - sol_network_forward uses the batch statistics of each convolution output as stored (for bf16: after
 *     rounding), keeps every layer output in the workspace and copies the logits to y.
 *
 * sol_network_backward: mean softmax cross-entropy of the logits left by the last forward against
 * labels (device int32 [n], each in [0, classes); any other value makes the loss NaN), then the full
 * backward pass.  *loss (device float, may be NULL) receives the loss.  Weight, gamma, beta and bias
 * gradients are fp32; activation gradients are stored in the network dtype; a tensor with several
 * consumers accumulates their contributions in descending layer order, the residual consumer of a
 * layer before its convolution.  x, workspace: as passed to the forward.  Deterministic.
 * The weight-gradient kernels run on a second stream owned by the network (created on the first call,
 * default priority, destroyed with the network) beside the chain of data gradients; everything is
 * ordered by events against `hip_stream`, so to the caller the call behaves as if it ran on that stream
 * alone.  Not capturable into a HIP graph.
 * SOL_ERR_UNSUPPORTED for inference networks. */
sol_status sol_network_backward(sol_network *net, const void *x, const int32_t *labels, float *loss,
                                void *workspace, size_t workspace_bytes, void *hip_stream);

/* v <- momentum * v + g ;  p <- p - lr * v  on every fp32 master parameter that received a gradient,
 * then re-packs the weights the kernels read. */
sol_status sol_network_sgd_step(sol_network *net, float lr, float momentum, void *hip_stream);

/* Device address and element count of a layer's fp32 training tensors inside the bound parameter buffer
 * (w and its gradient in framework layout [cout][cin][kh][kw]; the rest [cout]; mean / var: batch
 * statistics of the last forward, var biased). */
typedef enum sol_net_tensor {
    SOL_NT_W = 0, SOL_NT_GAMMA = 1, SOL_NT_BETA = 2, SOL_NT_BIAS = 3, SOL_NT_GRAD_W = 4, SOL_NT_GRAD_GAMMA = 5,
    SOL_NT_GRAD_BETA = 6, SOL_NT_GRAD_BIAS = 7, SOL_NT_MEAN = 8, SOL_NT_VAR = 9,
    SOL_NT_VEL_W = 10, SOL_NT_VEL_GAMMA = 11, SOL_NT_VEL_BETA = 12, SOL_NT_VEL_BIAS = 13   /* momentum buffers of the SGD step */
} sol_net_tensor;
sol_status sol_network_tensor(const sol_network *net, int layer, int which, float **ptr, size_t *count);

/* Device address (inside the workspace of the last forward) of the stored convolution output z of a
 * convolution layer with BN: the tensor its batch statistics were taken from (conv-output shape). */
sol_status sol_network_layer_preact(const sol_network *net, int layer, void *workspace, void **ptr);

/* Device address (inside the workspace of the last backward) of the gradient w.r.t. a layer's output. */
sol_status sol_network_layer_grad(const sol_network *net, int layer, void *workspace, void **ptr);

#ifdef __cplusplus
}
#endif
#endif /* SOL_MI355_H */

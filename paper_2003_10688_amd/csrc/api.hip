// C ABI of the library: argument validation, the single fused-layer entry points, and the network
// object (planner + executor).  Host code only; all device work is in conv_igemm.hip / fusion.hip.
#include <stdarg.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

#include "common.h"

namespace sol {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

static thread_local int g_tile_override = 0;   // debugging / sweeping aid of the calling thread, see sol_debug_set_conv_tile

static sol_status check_tensor(const sol_tensor_desc *d, const char *what) {
    SOL_REQUIRE(d, SOL_ERR_NULL, "%s descriptor is NULL", what);
    SOL_REQUIRE(d->dtype == SOL_F32 || d->dtype == SOL_BF16, SOL_ERR_DTYPE, "%s: unknown dtype %d", what, d->dtype);
    SOL_REQUIRE(d->n >= 0 && d->h > 0 && d->w > 0 && d->c > 0, SOL_ERR_SHAPE, "%s: bad shape [%d,%d,%d,%d]", what,
                d->n, d->h, d->w, d->c);
    SOL_REQUIRE((double)d->n * d->h * d->w * d->c < 2147483648.0, SOL_ERR_UNSUPPORTED, "%s: 2^31 elements or more", what);
    return SOL_OK;
}

static sol_status check_conv(const sol_conv_desc *cd) {
    SOL_REQUIRE(cd, SOL_ERR_NULL, "conv descriptor is NULL");
    SOL_REQUIRE(cd->cout > 0 && cd->cin > 0 && cd->kh > 0 && cd->kw > 0 && cd->sh > 0 && cd->sw > 0 && cd->ph >= 0 &&
                    cd->pw >= 0,
                SOL_ERR_SHAPE, "bad conv descriptor cout=%d cin=%d k=%dx%d s=%dx%d p=%dx%d", cd->cout, cd->cin, cd->kh,
                cd->kw, cd->sh, cd->sw, cd->ph, cd->pw);
    SOL_REQUIRE((double)cd->cout * cd->kh * cd->kw * cd->cin < 1073741824.0, SOL_ERR_UNSUPPORTED, "weight too large");
    return SOL_OK;
}

static sol_status check_pool(const sol_pool_desc *pd) {
    SOL_REQUIRE(pd, SOL_ERR_NULL, "pool descriptor is NULL");
    SOL_REQUIRE(pd->kind == SOL_POOL_MAX || pd->kind == SOL_POOL_AVG, SOL_ERR_SHAPE, "bad pool kind %d", pd->kind);
    SOL_REQUIRE(pd->kh > 0 && pd->kw > 0 && pd->sh > 0 && pd->sw > 0 && pd->ph >= 0 && pd->pw >= 0, SOL_ERR_SHAPE,
                "bad pool window k=%dx%d s=%dx%d p=%dx%d", pd->kh, pd->kw, pd->sh, pd->sw, pd->ph, pd->pw);
    SOL_REQUIRE(pd->ph < pd->kh && pd->pw < pd->kw, SOL_ERR_SHAPE, "pool padding must be smaller than the window");
    return SOL_OK;
}

static bool pool_is_fusable(const sol_pool_desc &p) {
    return p.kh == 2 && p.kw == 2 && p.sh == 2 && p.sw == 2 && p.ph == 0 && p.pw == 0;
}

#define SOL_TRY(expr)                   \
    do {                                \
        sol_status s_ = (expr);         \
        if (s_ != SOL_OK) return s_;    \
    } while (0)

// second operand set of a fused projection pair: y = act(scale * conv(x, w) + shift + scale2 * conv(x2, w2) + shift2)
struct PairOperand { const void *x2, *w2; const float *scale2, *shift2; int H2, W2, K2, Kp2, stride; };
// input side of a pre-activation convolution / of a convolution that reads a channel prefix of a wider tensor
struct InputSide { const float *pre_scale, *pre_shift; int ldx, cvalid; };   // NULL / NULL: no BN + ReLU; ldx 0: dense; cvalid 0: all channels real

// Shared by sol_conv2d_fused and the network executor.
static sol_status conv_fused_impl(const sol_tensor_desc &xd, const void *x, const sol_conv_desc &cd, const void *w,
                                  const float *scale, const float *shift, const void *res, int act,
                                  const sol_pool_desc *pool, void *y, int32_t *argmax, void *prepool, int tile,
                                  hipStream_t st, int ldy = 0,     // ldy: elements between output pixels in y, 0 = cout (dense)
                                  const PairOperand *pair = nullptr, const InputSide *ins = nullptr) {
    SOL_REQUIRE(cd.cin == xd.c, SOL_ERR_SHAPE, "conv cin %d != input channels %d", cd.cin, xd.c);
    SOL_REQUIRE(act == SOL_ACT_NONE || act == SOL_ACT_RELU, SOL_ERR_SHAPE, "bad activation %d", act);
    const int Ho = out_size(xd.h, cd.kh, cd.sh, cd.ph), Wo = out_size(xd.w, cd.kw, cd.sw, cd.pw);
    SOL_REQUIRE(xd.h + 2 * cd.ph >= cd.kh && xd.w + 2 * cd.pw >= cd.kw && Ho > 0 && Wo > 0, SOL_ERR_SHAPE,
                "filter %dx%d larger than padded input %dx%d", cd.kh, cd.kw, xd.h + 2 * cd.ph, xd.w + 2 * cd.pw);
    ConvArgs a;
    memset(static_cast<void *>(&a), 0, sizeof(a));
    a.N = xd.n; a.H = xd.h; a.W = xd.w; a.C = xd.c;
    a.Cout = cd.cout; a.R = cd.kh; a.S = cd.kw; a.sh = cd.sh; a.sw = cd.sw; a.ph = cd.ph; a.pw = cd.pw;
    a.Ho = Ho; a.Wo = Wo;
    a.Kp = packed_k(cd, xd.dtype);
    a.Ktot = cd.kh * cd.kw * cd.cin;
    a.act = act;
    a.res = res;
    a.pool = 0;
    a.Hy = Ho; a.Wy = Wo;
    if (pool && pool->kind != SOL_POOL_NONE) {
        SOL_TRY(check_pool(pool));
        if (pool_is_fusable(*pool)) {
            a.pool = pool->kind == SOL_POOL_MAX ? 1 : 2;
            a.Hy = Ho / 2; a.Wy = Wo / 2;
            SOL_REQUIRE(a.Hy > 0 && a.Wy > 0, SOL_ERR_SHAPE, "conv output %dx%d too small for a 2x2 pool", Ho, Wo);
        } else {
            SOL_REQUIRE(stem_pool_applies(a, xd.dtype, *pool), SOL_ERR_UNSUPPORTED,
                        "a pool fused into the convolution is 2x2 stride 2 unpadded, or a 3x3 stride-2 pad-1 max pool behind a bf16 "
                        "7x7 stride-2 convolution of 3 channels with 64 filters, ReLU and no residual; run sol_pool separately");
            SOL_REQUIRE(!argmax && !prepool, SOL_ERR_UNSUPPORTED, "the fused stem pool stores neither winners nor the pre-pool tensor");
            a.pool = 3;
            a.Hy = out_size(Ho, 3, 2, 1); a.Wy = out_size(Wo, 3, 2, 1);
        }
    }
    a.ldy = cd.cout;
    if (ldy != 0 && ldy != cd.cout) {
        SOL_REQUIRE(ldy > cd.cout && ldy % 8 == 0 && cd.cout % 8 == 0, SOL_ERR_SHAPE,
                    "output pitch %d: a multiple of 8 above cout (%d, itself a multiple of 8)", ldy, cd.cout);
        SOL_REQUIRE(a.pool == 0, SOL_ERR_UNSUPPORTED, "a convolution with a fused pool writes a dense output");
        a.ldy = ldy;
    }
    SOL_REQUIRE((double)xd.n * Ho * Wo * a.ldy < 2147483648.0, SOL_ERR_UNSUPPORTED, "output spans 2^31 elements or more");
    a.ldx = xd.c;
    a.Cvalid = xd.c;
    if (ins) {
        SOL_REQUIRE((ins->pre_scale == nullptr) == (ins->pre_shift == nullptr), SOL_ERR_NULL, "input-side scale and shift come together");
        SOL_REQUIRE(aligned16(ins->pre_scale) && aligned16(ins->pre_shift), SOL_ERR_ALIGN, "device pointers must be 16-byte aligned");
        if (ins->ldx != 0 && ins->ldx != xd.c) {
            SOL_REQUIRE(ins->ldx > xd.c && (ins->ldx * dtype_size(xd.dtype)) % 16 == 0, SOL_ERR_SHAPE,
                        "input pitch %d: above the channel count %d, pixels 16-byte aligned", ins->ldx, xd.c);
            SOL_REQUIRE((double)xd.n * xd.h * xd.w * ins->ldx < 2147483648.0, SOL_ERR_UNSUPPORTED, "input spans 2^31 elements or more");
            a.ldx = ins->ldx;
        }
        if (ins->cvalid != 0) {
            SOL_REQUIRE(ins->cvalid > 0 && ins->cvalid <= xd.c, SOL_ERR_SHAPE, "%d valid input channels of %d", ins->cvalid, xd.c);
            a.Cvalid = ins->cvalid;
        }
        a.pre_scale = ins->pre_scale; a.pre_shift = ins->pre_shift;
        SOL_REQUIRE(!(pool && a.pool == 3) && !pair, SOL_ERR_UNSUPPORTED, "the fused stem pair and the projection pair take a plain dense input");
    }
    if (xd.n == 0) return SOL_OK;
    SOL_REQUIRE(x && w && y, SOL_ERR_NULL, "x, w_packed and y must not be NULL");
    SOL_REQUIRE(aligned16(x) && aligned16(w) && aligned16(y) && aligned16(scale) && aligned16(shift) && aligned16(res) &&
                    aligned16(argmax) && aligned16(prepool),
                SOL_ERR_ALIGN, "device pointers must be 16-byte aligned");
    a.x = x; a.w = w; a.scale = scale; a.shift = shift; a.y = y;
    const bool quad = a.pool == 1 || a.pool == 2;
    a.argmax = a.pool == 1 ? argmax : nullptr;
    a.prepool = quad ? prepool : nullptr;
    a.P = quad ? xd.n * a.Hy * a.Wy * 4 : xd.n * Ho * Wo;
    a.dw = FastDiv((uint32_t)(quad ? a.Wy : Wo));
    a.dh = FastDiv((uint32_t)(quad ? a.Hy : Ho));
    if (a.pool == 3) return launch_conv_stem_pool(a, st);   // one kernel, no tile choice
    if (pair) {
        SOL_REQUIRE(res == nullptr && pair_applies(a, xd.dtype, pair->H2, pair->W2, pair->K2, pair->Kp2, pair->stride), SOL_ERR_UNSUPPORTED,
                    "a fused projection pair is two bf16 unpadded 1x1 convolutions over multiples of 64 channels");
        SOL_REQUIRE(pair->x2 && pair->w2 && aligned16(pair->x2) && aligned16(pair->w2), SOL_ERR_NULL, "pair operands");
        return launch_conv_pair(a, pair->x2, pair->w2, pair->scale2, pair->shift2, pair->H2, pair->W2, pair->K2, pair->Kp2, pair->stride, st);
    }
    return launch_conv(a, xd.dtype, tile, st);
}

static sol_status pool_impl(const sol_tensor_desc &xd, const void *x, const sol_pool_desc &pd, void *y, int32_t *argmax,
                            hipStream_t st) {
    SOL_TRY(check_pool(&pd));
    SOL_REQUIRE(xd.h + 2 * pd.ph >= pd.kh && xd.w + 2 * pd.pw >= pd.kw, SOL_ERR_SHAPE, "pool window larger than padded input");
    if (xd.n == 0) return SOL_OK;
    SOL_REQUIRE(x && y, SOL_ERR_NULL, "x and y must not be NULL");
    SOL_REQUIRE(aligned16(x) && aligned16(y) && aligned16(argmax), SOL_ERR_ALIGN, "device pointers must be 16-byte aligned");
    PoolArgs a;
    a.x = x; a.y = y; a.argmax = argmax;
    a.N = xd.n; a.H = xd.h; a.W = xd.w; a.C = xd.c;
    a.Ho = out_size(xd.h, pd.kh, pd.sh, pd.ph); a.Wo = out_size(xd.w, pd.kw, pd.sw, pd.pw);
    a.kh = pd.kh; a.kw = pd.kw; a.sh = pd.sh; a.sw = pd.sw; a.ph = pd.ph; a.pw = pd.pw;
    a.kind = pd.kind; a.count_pad = pd.count_pad;
    return launch_pool(a, xd.dtype, st);
}

static size_t dw_weight_bytes(int c, int kh, int kw, int dt) { return round_up((size_t)c * kh * kw * dtype_size(dt), 16); }

// Shared by sol_dwconv2d_fused and the network executor.
static sol_status dwconv_impl(const sol_tensor_desc &xd, const void *x, const sol_conv_desc &cd, const void *w,
                              const float *scale, const float *shift, const void *res, int act, void *y, hipStream_t st) {
    SOL_REQUIRE(cd.cin == xd.c && cd.cout == xd.c, SOL_ERR_SHAPE, "depthwise conv: cin %d and cout %d must both equal the input channels %d",
                cd.cin, cd.cout, xd.c);
    SOL_REQUIRE(act == SOL_ACT_NONE || act == SOL_ACT_RELU, SOL_ERR_SHAPE, "bad activation %d", act);
    SOL_REQUIRE(cd.kh * cd.kw <= 1024, SOL_ERR_UNSUPPORTED, "depthwise filter %dx%d too large", cd.kh, cd.kw);
    const int Ho = out_size(xd.h, cd.kh, cd.sh, cd.ph), Wo = out_size(xd.w, cd.kw, cd.sw, cd.pw);
    SOL_REQUIRE(xd.h + 2 * cd.ph >= cd.kh && xd.w + 2 * cd.pw >= cd.kw && Ho > 0 && Wo > 0, SOL_ERR_SHAPE,
                "filter %dx%d larger than padded input %dx%d", cd.kh, cd.kw, xd.h + 2 * cd.ph, xd.w + 2 * cd.pw);
    SOL_REQUIRE((double)xd.n * Ho * Wo * xd.c < 2147483648.0, SOL_ERR_UNSUPPORTED, "output has 2^31 elements or more");
    if (xd.n == 0) return SOL_OK;
    SOL_REQUIRE(x && w && y, SOL_ERR_NULL, "x, w_packed and y must not be NULL");
    SOL_REQUIRE(aligned16(x) && aligned16(w) && aligned16(y) && aligned16(scale) && aligned16(shift) && aligned16(res),
                SOL_ERR_ALIGN, "device pointers must be 16-byte aligned");
    DwArgs a;
    a.x = x; a.w = w; a.res = res; a.scale = scale; a.shift = shift; a.y = y;
    a.N = xd.n; a.H = xd.h; a.W = xd.w; a.C = xd.c; a.Ho = Ho; a.Wo = Wo;
    a.kh = cd.kh; a.kw = cd.kw; a.sh = cd.sh; a.sw = cd.sw; a.ph = cd.ph; a.pw = cd.pw;
    a.act = act;
    return launch_dwconv(a, xd.dtype, st);
}

// ---- network ---------------------------------------------------------------------------------------
struct LayerPlan {
    sol_layer L;
    sol_tensor_desc in, out;        // input / stored output
    sol_tensor_desc conv_out;       // CONV: convolution output (before any pool)
    sol_conv_desc cd;               // CONV / LINEAR (as 1x1)
    int src, res;                   // resolved producer indices, -1 = network input
    bool fuse_pool, split_pool;     // CONV with pool: fused into the epilogue, or run as a second launch
    bool absorbs_next, elided;      // a stem convolution that also computes the max-pool layer behind it / that pool layer
    int nuse;                       // how many layer inputs (src or res) read this layer's output
    int cout_real, cin_real;        // CONV: channel counts of the caller's weights when the plan padded cd.cout / cd.cin (else 0)
    int concat_into, concat_off;    // CONV: writes its output as channels concat_off.. of that CONCAT layer's buffer (-1: own buffer)
    bool prealloc;                  // CONCAT: buffer laid out when its first in-place producer ran
    int pair;                       // CONV: index of the projection convolution this launch also computes (-1: none)
    int block_c1, block_c2;         // CONV (last 1x1 of a bottleneck): the reduce and 3x3 convolutions that one depth-first launch can compute with it (-1: none)
    int block_c3;                   // CONV (reduce / 3x3 of such a bottleneck): that last convolution (-1: none)
    bool use_block;                 // on the last convolution: the plan runs the bottleneck as one launch (heuristic or sol_network_autotune)
    int xr_next, xr_from;           // CONV (last 1x1 of a bottleneck): the next bottleneck's first 1x1, which the same launch can compute (conv_xr.hip); on that layer: the former (-1: none)
    bool use_xr;                    // on the former: the plan runs the two as one launch
    bool pre_bn, pre_set;           // CONV: BN + ReLU on the input side; its folded constants have been set
    size_t pre_scale_off, pre_shift_off;
    int ldx;                        // CONV: input pixel pitch when the input is a channel prefix of a dense-block buffer (0: dense)
    int chain_owner;                // CONCAT: last CONCAT of the dense chain whose buffer this layer is a prefix of (-1: none; itself for the last)
    bool part_inplace[2];           // CONCAT: src / res part already sits in the output buffer when the layer runs
    int fused_into;                 // index of the layer whose launch produces this layer's output (itself unless elided)
    bool no_buffer;                 // elided, and nobody allocates an output for it either
    size_t w_off, scale_off, shift_off;
    size_t out_off, tmp_off;        // workspace offsets; out_off unused for the last layer
    int last_use;
    bool params_set;
    int tile;                       // CONV / LINEAR: kernel + tile id chosen by sol_network_autotune (T_AUTO: shape heuristic)
    int tile_dgrad;                 // training: the same for the data-gradient convolution
    // training networks only
    size_t wT_off, master_off, vel_off, grad_off, vec_off;   // parameter buffer: flipped pack, fp32 master / velocity / gradient, per-channel arrays
    size_t z_off, dact_off, arg_off;                          // workspace: conv output before BN, gradient of the output, pool winners
    size_t wpart_off;                                         // workspace: split partials of this layer's weight gradient
    size_t dzl_off;                                           // workspace: this layer's dz (kept until its weight gradient has run)
    bool has_grad, need_dgrad, src_first, res_first, dilate;
    sol_conv_desc dcd;                                        // data-gradient as a stride-1 convolution ...
    sol_tensor_desc dzd;                                      // ... over dz (zero-inserted when the forward stride is > 1)
    float eps;
};

// per-channel fp32 arrays of a trainable layer, each padded to 256 bytes
enum { VEC_GAMMA, VEC_BETA, VEC_BIAS, VEC_V_GAMMA, VEC_V_BETA, VEC_V_BIAS, VEC_G_GAMMA, VEC_G_BETA, VEC_G_BIAS, VEC_MEAN,
       VEC_VAR, VEC_INVSTD, VEC_COUNT };

}  // namespace sol

struct sol_network {
    std::vector<sol::LayerPlan> layers;
    sol_tensor_desc input;
    int training, keep;
    size_t param_bytes, ws_bytes;
    unsigned char *params;
    size_t params_size;
    size_t dz_off, dil_off, part_off, loss_off;   // training: shared scratch inside the workspace
    size_t dz_bytes, dil_bytes;
    // Backward pass: the weight gradient of a layer needs only dz and the stored input, and nothing but the final
    // reduction needs its result, while the chain dz -> data gradient -> next layer is a string of short,
    // latency-bound launches.  The weight-gradient kernels therefore go to a stream of the library's own and overlap
    // that chain (default priority; created on the first backward call, on its device).  Cross-stream events cost
    // the main chain several microseconds each, so every layer keeps its dz in a buffer of its own and the side
    // stream is handed the weight gradients of a few layers at a time behind one event.
    hipStream_t side = nullptr;
    hipEvent_t ev_ready = nullptr, ev_join = nullptr;
    ~sol_network() {
        if (ev_ready) (void)hipEventDestroy(ev_ready);
        if (ev_join) (void)hipEventDestroy(ev_join);
        if (side) (void)hipStreamDestroy(side);
    }
};

namespace sol {

// first-fit allocator over a growing arena, used at plan time to lay activations out in the workspace
struct Arena {
    struct Blk { size_t off, size; bool free; };
    std::vector<Blk> blks;
    size_t top = 0;
    size_t alloc(size_t bytes) {
        bytes = round_up(std::max<size_t>(bytes, 256), 256);
        for (size_t i = 0; i < blks.size(); i++)
            if (blks[i].free && blks[i].size >= bytes) {
                if (blks[i].size > bytes) {
                    Blk rest{blks[i].off + bytes, blks[i].size - bytes, true};
                    blks[i].size = bytes;
                    blks.insert(blks.begin() + i + 1, rest);
                }
                blks[i].free = false;
                return blks[i].off;
            }
        if (!blks.empty() && blks.back().free) {   // grow the trailing free block
            blks.back().size = bytes; blks.back().free = false;
            top = blks.back().off + bytes;
            return blks.back().off;
        }
        blks.push_back(Blk{top, bytes, false});
        top += bytes;
        return blks.back().off;
    }
    void release(size_t off) {
        for (size_t i = 0; i < blks.size(); i++)
            if (blks[i].off == off) {
                blks[i].free = true;
                if (i + 1 < blks.size() && blks[i + 1].free) { blks[i].size += blks[i + 1].size; blks.erase(blks.begin() + i + 1); }
                if (i > 0 && blks[i - 1].free) { blks[i - 1].size += blks[i].size; blks.erase(blks.begin() + i); }
                return;
            }
    }
};

static size_t tensor_bytes(const sol_tensor_desc &d) { return (size_t)d.n * d.h * d.w * d.c * dtype_size(d.dtype); }

// Training: which layers receive a gradient, in which order a tensor's consumers contribute to it
// (descending consumer index, residual before data-gradient), and the extra workspace.
static sol_status plan_training(sol_network *net, Arena &ar) {
    const int nl = (int)net->layers.size();
    const sol_tensor_desc &lo = net->layers[nl - 1].out;
    SOL_REQUIRE(lo.h == 1 && lo.w == 1, SOL_ERR_UNSUPPORTED, "training: the last layer must produce [n,1,1,classes] logits");
    std::vector<char> seen(nl, 0);
    seen[nl - 1] = 1;
    size_t dz_max = 0, dil_max = 0, part_max = 0;
    for (int i = nl - 1; i >= 0; i--) {
        LayerPlan &lp = net->layers[i];
        lp.has_grad = seen[i];
        lp.dact_off = ar.alloc(tensor_bytes(lp.out));
        const int kind = lp.L.kind;
        if (kind == SOL_LAYER_POOL && lp.L.pool.kind == SOL_POOL_MAX)
            lp.arg_off = ar.alloc((size_t)lp.out.n * lp.out.h * lp.out.w * lp.out.c * 4);
        if (kind == SOL_LAYER_CONV || kind == SOL_LAYER_LINEAR) {
            if (kind == SOL_LAYER_CONV && lp.L.has_bn) lp.z_off = ar.alloc(tensor_bytes(lp.conv_out));
            dz_max = std::max(dz_max, tensor_bytes(lp.conv_out));
            int ns; size_t pf;
            wgrad_plan(lp.in, lp.cd, lp.conv_out.h, lp.conv_out.w, &ns, &pf);
            lp.wpart_off = ar.alloc(pf * 4);       // kept until the end of the backward pass: all layers' partials are added by one launch
            lp.dzl_off = ar.alloc(std::max<size_t>(tensor_bytes(lp.conv_out), 256));
            const int rows = lp.conv_out.n * lp.conv_out.h * lp.conv_out.w;
            part_max = std::max(part_max, std::max(pf * 4, (size_t)col_reduce_chunks(rows, nullptr) * 2 * lp.cd.cout * 4));
            if (lp.dilate) dil_max = std::max(dil_max, tensor_bytes(lp.dzd));
        }
        if (!seen[i]) continue;
        if (lp.res >= 0) { lp.res_first = !seen[lp.res]; seen[lp.res] = 1; }
        if (lp.src >= 0) { lp.src_first = !seen[lp.src]; seen[lp.src] = 1; lp.need_dgrad = true; }
    }
    net->dz_off = ar.alloc(dz_max);
    net->dil_off = ar.alloc(dil_max);
    net->dz_bytes = dz_max; net->dil_bytes = dil_max;
    net->part_off = ar.alloc(part_max);
    net->loss_off = ar.alloc(((size_t)net->input.n + 1) * 4);
    return SOL_OK;
}

// can this convolution layer run fused with the 3x3 stride-2 max pool `p` behind it (conv_stem_pool_kernel)?
static bool stem_pool_plan_ok(const sol_tensor_desc &in, const sol_conv_desc &cd, const sol_layer &L, const sol_pool_desc &p) {
    ConvArgs a;
    memset(static_cast<void *>(&a), 0, sizeof(a));
    a.N = in.n; a.H = in.h; a.W = in.w; a.C = in.c;
    a.Cout = cd.cout; a.R = cd.kh; a.S = cd.kw; a.sh = cd.sh; a.sw = cd.sw; a.ph = cd.ph; a.pw = cd.pw;
    a.Kp = packed_k(cd, in.dtype);
    a.act = L.act;
    return L.res < 0 && stem_pool_applies(a, in.dtype, p);
}

static sol_status plan_network(sol_network *net, const sol_layer *layers, int n_layers) {
    const int dt = net->input.dtype;
    net->layers.resize(n_layers);
    size_t poff = 0;
    // Channel padding (the paper's layout selection, Sec. III-A: feed every layer the layout it is fastest with).  The
    // fast convolution kernels fetch the reduction in 64-byte runs of channels; a producer with, say, 16 or 48
    // filters would push every convolution behind it onto the element-gather path (5-10x slower).  Such a
    // convolution, when only convolutions read it, stores its output with the channel count rounded up to 32: its
    // extra filters and its consumers' extra input channels are zero weights, so every real value is unchanged.
    std::vector<int> pad_to(n_layers, 0);
    if (!net->training && !net->keep)
        for (int i = 0; i + 1 < n_layers; i++) {
            const sol_layer &L = layers[i];
            if (L.kind != SOL_LAYER_CONV || L.pool.kind != SOL_POOL_NONE || L.res >= 0 || L.conv.cout < 16 || L.conv.cout % 32 == 0) continue;
            int readers = 0;
            bool ok = true;
            for (int j = i + 1; j < n_layers; j++) {
                const int sj = layers[j].src == -1 ? j - 1 : layers[j].src;
                if (sj == i) { readers++; ok = ok && layers[j].kind == SOL_LAYER_CONV; }
                if (layers[j].res == i && (layers[j].kind == SOL_LAYER_CONV || layers[j].kind == SOL_LAYER_DWCONV ||
                                           layers[j].kind == SOL_LAYER_CONCAT)) ok = false;
            }
            if (ok && readers > 0) pad_to[i] = (int)round_up((size_t)L.conv.cout, 32);
        }
    for (int i = 0; i < n_layers; i++) {
        LayerPlan &lp = net->layers[i];
        memset(&lp, 0, sizeof(lp));
        lp.L = layers[i];
        const sol_layer &L = lp.L;
        SOL_REQUIRE(L.src >= -1 && L.src < i, SOL_ERR_SHAPE, "layer %d: src %d must name an earlier layer", i, L.src);
        lp.src = L.src == -1 ? i - 1 : L.src;
        lp.res = -1;
        lp.concat_into = -1;
        lp.pair = -1;
        lp.block_c1 = lp.block_c2 = lp.block_c3 = -1;
        lp.xr_next = lp.xr_from = -1;
        lp.chain_owner = -1;
        lp.fused_into = i;
        lp.in = lp.src < 0 ? net->input : net->layers[lp.src].out;
        lp.out = lp.in;
        lp.last_use = i;
        switch (L.kind) {
            case SOL_LAYER_CONV: {
                lp.cd = L.conv;
                lp.cd.cin = lp.in.c;
                lp.pre_bn = L.pre_bn != 0;
                SOL_REQUIRE(!(lp.pre_bn && net->training), SOL_ERR_UNSUPPORTED, "layer %d: input-side batch-norm is inference-only", i);
                if (lp.src >= 0 && net->layers[lp.src].cout_real) lp.cin_real = net->layers[lp.src].cout_real;
                if (pad_to[i]) { lp.cout_real = lp.cd.cout; lp.cd.cout = pad_to[i]; }
                SOL_TRY(check_conv(&lp.cd));
                SOL_REQUIRE(lp.in.h + 2 * lp.cd.ph >= lp.cd.kh && lp.in.w + 2 * lp.cd.pw >= lp.cd.kw, SOL_ERR_SHAPE,
                            "layer %d: filter larger than padded input", i);
                lp.conv_out = lp.in;
                lp.conv_out.h = out_size(lp.in.h, lp.cd.kh, lp.cd.sh, lp.cd.ph);
                lp.conv_out.w = out_size(lp.in.w, lp.cd.kw, lp.cd.sw, lp.cd.pw);
                lp.conv_out.c = lp.cd.cout;
                lp.out = lp.conv_out;
                SOL_REQUIRE(!(net->training && L.pool.kind != SOL_POOL_NONE), SOL_ERR_UNSUPPORTED,
                            "layer %d: training networks take the pool as a layer of its own", i);
                if (L.pool.kind != SOL_POOL_NONE) {
                    SOL_TRY(check_pool(&L.pool));
                    lp.fuse_pool = pool_is_fusable(L.pool) || stem_pool_plan_ok(lp.in, lp.cd, L, L.pool);
                    lp.split_pool = !lp.fuse_pool;
                    SOL_REQUIRE(lp.conv_out.h + 2 * L.pool.ph >= L.pool.kh && lp.conv_out.w + 2 * L.pool.pw >= L.pool.kw,
                                SOL_ERR_SHAPE, "layer %d: pool window larger than its input", i);
                    lp.out.h = out_size(lp.conv_out.h, L.pool.kh, L.pool.sh, L.pool.ph);
                    lp.out.w = out_size(lp.conv_out.w, L.pool.kw, L.pool.sw, L.pool.pw);
                }
                if (L.res >= 0) {
                    SOL_REQUIRE(L.res < i, SOL_ERR_SHAPE, "layer %d: residual %d must name an earlier layer", i, L.res);
                    const sol_tensor_desc &r = net->layers[L.res].out;
                    SOL_REQUIRE(r.n == lp.conv_out.n && r.h == lp.conv_out.h && r.w == lp.conv_out.w && r.c == lp.conv_out.c,
                                SOL_ERR_SHAPE, "layer %d: residual shape [%d,%d,%d,%d] != conv output [%d,%d,%d,%d]", i, r.n,
                                r.h, r.w, r.c, lp.conv_out.n, lp.conv_out.h, lp.conv_out.w, lp.conv_out.c);
                    lp.res = L.res;
                }
                break;
            }
            case SOL_LAYER_DWCONV: {
                SOL_REQUIRE(!net->training, SOL_ERR_UNSUPPORTED, "layer %d: depthwise convolutions are inference-only", i);
                SOL_REQUIRE(L.conv.cout == 0 || L.conv.cout == lp.in.c, SOL_ERR_SHAPE,
                            "layer %d: a depthwise convolution keeps the channel count (%d), cout is %d", i, lp.in.c, L.conv.cout);
                SOL_REQUIRE(L.pool.kind == SOL_POOL_NONE, SOL_ERR_UNSUPPORTED,
                            "layer %d: a pool behind a depthwise convolution is a layer of its own", i);
                lp.cd = L.conv;
                lp.cd.cin = lp.cd.cout = lp.in.c;
                SOL_TRY(check_conv(&lp.cd));
                SOL_REQUIRE(lp.in.h + 2 * lp.cd.ph >= lp.cd.kh && lp.in.w + 2 * lp.cd.pw >= lp.cd.kw, SOL_ERR_SHAPE,
                            "layer %d: filter larger than padded input", i);
                lp.conv_out = lp.in;
                lp.conv_out.h = out_size(lp.in.h, lp.cd.kh, lp.cd.sh, lp.cd.ph);
                lp.conv_out.w = out_size(lp.in.w, lp.cd.kw, lp.cd.sw, lp.cd.pw);
                lp.out = lp.conv_out;
                if (L.res >= 0) {
                    SOL_REQUIRE(L.res < i, SOL_ERR_SHAPE, "layer %d: residual %d must name an earlier layer", i, L.res);
                    const sol_tensor_desc &r = net->layers[L.res].out;
                    SOL_REQUIRE(r.n == lp.out.n && r.h == lp.out.h && r.w == lp.out.w && r.c == lp.out.c, SOL_ERR_SHAPE,
                                "layer %d: residual shape [%d,%d,%d,%d] != output [%d,%d,%d,%d]", i, r.n, r.h, r.w, r.c,
                                lp.out.n, lp.out.h, lp.out.w, lp.out.c);
                    lp.res = L.res;
                }
                break;
            }
            case SOL_LAYER_POOL:
                SOL_TRY(check_pool(&L.pool));
                SOL_REQUIRE(lp.in.h + 2 * L.pool.ph >= L.pool.kh && lp.in.w + 2 * L.pool.pw >= L.pool.kw, SOL_ERR_SHAPE,
                            "layer %d: pool window larger than its input", i);
                lp.out.h = out_size(lp.in.h, L.pool.kh, L.pool.sh, L.pool.ph);
                lp.out.w = out_size(lp.in.w, L.pool.kw, L.pool.sw, L.pool.pw);
                break;
            case SOL_LAYER_GAP:
                lp.out.h = lp.out.w = 1;
                break;
            case SOL_LAYER_CONCAT: {
                SOL_REQUIRE(!net->training, SOL_ERR_UNSUPPORTED, "layer %d: concatenations are inference-only", i);
                SOL_REQUIRE(lp.src >= 0 && L.res >= 0 && L.res < i && L.res != lp.src, SOL_ERR_SHAPE,
                            "layer %d: a concatenation joins two different earlier layers (src %d, res %d)", i, lp.src, L.res);
                const sol_tensor_desc &b = net->layers[L.res].out;
                SOL_REQUIRE(b.n == lp.in.n && b.h == lp.in.h && b.w == lp.in.w, SOL_ERR_SHAPE,
                            "layer %d: concatenation of [%d,%d,%d,%d] and [%d,%d,%d,%d]", i, lp.in.n, lp.in.h, lp.in.w, lp.in.c, b.n,
                            b.h, b.w, b.c);
                lp.res = L.res;
                lp.out.c = lp.in.c + b.c;
                break;
            }
            case SOL_LAYER_LINEAR:
                SOL_REQUIRE(L.out_features > 0, SOL_ERR_SHAPE, "layer %d: out_features %d", i, L.out_features);
                SOL_REQUIRE(lp.in.h == 1 && lp.in.w == 1, SOL_ERR_UNSUPPORTED,
                            "layer %d: linear needs a [n,1,1,c] input (put a global average pool in front)", i);
                lp.cd = sol_conv_desc{L.out_features, lp.in.c, 1, 1, 1, 1, 0, 0};
                lp.conv_out = lp.in;
                lp.conv_out.c = L.out_features;
                lp.out = lp.conv_out;
                break;
            default: SOL_FAIL(SOL_ERR_SHAPE, "layer %d: unknown kind %d", i, L.kind);
        }
        SOL_TRY(check_tensor(&lp.out, "layer output"));
        if (L.kind == SOL_LAYER_DWCONV) {
            lp.w_off = poff; poff += round_up(dw_weight_bytes(lp.cd.cout, lp.cd.kh, lp.cd.kw, dt), 256);
            lp.scale_off = poff; poff += round_up((size_t)lp.cd.cout * 4, 256);
            lp.shift_off = poff; poff += round_up((size_t)lp.cd.cout * 4, 256);
        }
        if (L.kind == SOL_LAYER_CONV || L.kind == SOL_LAYER_LINEAR) {
            lp.w_off = poff; poff += round_up(sol_packed_weight_bytes(&lp.cd, (sol_dtype)dt), 256);
            lp.scale_off = poff; poff += round_up((size_t)lp.cd.cout * 4, 256);
            lp.shift_off = poff; poff += round_up((size_t)lp.cd.cout * 4, 256);
            if (lp.pre_bn) {        // room for the channel count rounded up to one reduction chunk (a prefix of a dense-block buffer)
                lp.pre_scale_off = poff; poff += round_up((size_t)(lp.cd.cin + 64) * 4, 256);
                lp.pre_shift_off = poff; poff += round_up((size_t)(lp.cd.cin + 64) * 4, 256);
            }
            if (net->training) {
                const size_t wb = round_up((size_t)lp.cd.cout * lp.cd.cin * lp.cd.kh * lp.cd.kw * 4, 256);
                lp.master_off = poff; poff += wb;
                lp.vel_off = poff; poff += wb;
                lp.grad_off = poff; poff += wb;
                lp.vec_off = poff; poff += VEC_COUNT * round_up((size_t)lp.cd.cout * 4, 256);
                if (lp.src >= 0) {
                    SOL_REQUIRE(lp.cd.ph < lp.cd.kh && lp.cd.pw < lp.cd.kw, SOL_ERR_UNSUPPORTED,
                                "layer %d: training needs padding smaller than the filter", i);
                    // dx = stride-1 convolution of the zero-inserted dz with the flipped filter, padding k-1-p
                    lp.dcd = sol_conv_desc{lp.cd.cin, lp.cd.cout, lp.cd.kh, lp.cd.kw, 1, 1, lp.cd.kh - 1 - lp.cd.ph,
                                           lp.cd.kw - 1 - lp.cd.pw};
                    lp.dzd = lp.conv_out;
                    lp.dzd.h = lp.in.h + 2 * lp.cd.ph - lp.cd.kh + 1;
                    lp.dzd.w = lp.in.w + 2 * lp.cd.pw - lp.cd.kw + 1;
                    lp.dilate = lp.cd.sh > 1 || lp.cd.sw > 1;
                    SOL_TRY(check_tensor(&lp.dzd, "zero-inserted gradient"));
                    lp.wT_off = poff; poff += round_up(sol_packed_weight_bytes(&lp.dcd, (sol_dtype)dt), 256);
                }
            }
        }
        if (lp.src >= 0) { net->layers[lp.src].last_use = i; net->layers[lp.src].nuse++; }
        if (lp.res >= 0) { net->layers[lp.res].last_use = std::max(net->layers[lp.res].last_use, i); net->layers[lp.res].nuse++; }
    }
    net->param_bytes = poff;

    // Dense chains.  A CONCAT whose src is the CONCAT in front of it extends that tensor by new channels (the dense
    // blocks of a DenseNet-shaped list).  When every intermediate join is read only by unpadded 1x1 convolutions and by
    // its extension, the whole chain shares ONE buffer of the final width: producers write their slices into it, the
    // 1x1 convolutions read a channel prefix of it (pixel pitch = final width, reduction rounded up to whole chunks with
    // the extra channels masked to zero), and nothing is ever copied but the block input.
    if (!net->training && !net->keep) {
        const int chunk = dt == SOL_BF16 ? 64 : 32;
        std::vector<int> ext(n_layers, -1), is_ext(n_layers, 0);
        for (int j = 0; j < n_layers; j++) {
            if (net->layers[j].L.kind != SOL_LAYER_CONCAT) continue;
            int e = -1;
            bool ok = true;
            for (int t = j + 1; t < n_layers; t++) {
                const LayerPlan &r = net->layers[t];
                if (r.src != j && r.res != j) continue;
                if (r.L.kind == SOL_LAYER_CONCAT && r.src == j && r.res != j && e < 0) e = t;
                else if (r.L.kind == SOL_LAYER_CONV && r.src == j && r.res != j && r.cd.kh == 1 && r.cd.kw == 1 && r.cd.ph == 0 && r.cd.pw == 0) {}
                else ok = false;
            }
            if (ok && e >= 0) { ext[j] = e; is_ext[e] = 1; }
        }
        for (int j = 0; j < n_layers; j++) {
            if (ext[j] < 0 || is_ext[j]) continue;                       // heads only
            std::vector<int> mem;
            for (int k = j; k >= 0; k = ext[k]) mem.push_back(k);
            const int last = mem.back(), ctot = net->layers[last].out.c;
            bool ok = last + 1 < n_layers && ctot % 8 == 0 && (ctot * dtype_size(dt)) % 16 == 0;
            for (int k : mem) ok = ok && net->layers[k].out.c % 8 == 0 && net->layers[k].in.c % 8 == 0;
            if (!ok) continue;
            for (int k : mem) {
                net->layers[k].chain_owner = last;
                if (k == last) continue;
                for (int t = k + 1; t < n_layers; t++) {                  // its readers fetch a prefix of the shared buffer
                    LayerPlan &r = net->layers[t];
                    if (r.L.kind != SOL_LAYER_CONV || r.src != k) continue;
                    r.ldx = ctot;
                    const int cpad = std::min((int)round_up((size_t)r.cd.cin, chunk), ctot);
                    if (cpad != r.cd.cin) { r.cin_real = r.cd.cin; r.cd.cin = cpad; }
                }
            }
        }
    }

    // Depth-first pair (the paper's layer-chain fusion, Sec. III-A / IV): a stem convolution whose output feeds
    // nothing but the max-pool layer behind it runs in one kernel with that pool; the convolution's output, the
    // largest tensor of the list, never exists.  Not when every activation is kept for the caller or for training.
    if (!net->training && !net->keep)
        for (int i = 0; i + 1 < n_layers; i++) {
            LayerPlan &c = net->layers[i], &q = net->layers[i + 1];
            if (c.L.kind == SOL_LAYER_CONV && c.L.pool.kind == SOL_POOL_NONE && q.L.kind == SOL_LAYER_POOL && q.src == i &&
                c.last_use == i + 1 && stem_pool_plan_ok(c.in, c.cd, c.L, q.L.pool)) {
                c.absorbs_next = true;
                q.elided = true;
                q.fused_into = i;
            }
        }

    // Projection pair: the 1x1 shortcut convolution of a block whose only reader is the residual input of the
    // block's last 1x1 convolution runs inside that convolution's launch (both over 64 channels: conv_pair.hip);
    // its output, as large as the block output, is neither written nor read back.
    if (!net->training && !net->keep && dt == SOL_BF16)
        for (int i = 0; i < n_layers; i++) {
            LayerPlan &c = net->layers[i];
            if (c.L.kind != SOL_LAYER_CONV || c.res < 0 || c.L.pool.kind != SOL_POOL_NONE || c.cout_real || c.cin_real || c.pre_bn || c.ldx) continue;
            LayerPlan &p = net->layers[c.res];
            const auto pointwise = [](const LayerPlan &l) {      // unpadded 1x1 over a multiple of 64 channels
                return l.cd.kh == 1 && l.cd.kw == 1 && l.cd.ph == 0 && l.cd.pw == 0 && l.cd.cin % 64 == 0 && l.cd.sh == l.cd.sw;
            };
            if (p.L.kind == SOL_LAYER_CONV && p.L.act == SOL_ACT_NONE && p.res < 0 && p.L.pool.kind == SOL_POOL_NONE && p.nuse == 1 &&
                !p.elided && !p.absorbs_next && !p.cout_real && !p.cin_real && !p.pre_bn && !p.ldx && pointwise(p) && pointwise(c) && c.cd.sh == 1 &&
                c.cd.cout % 8 == 0 && c.src != c.res && tensor_bytes(p.in) < (1u << 31) && tensor_bytes(c.in) < (1u << 31)) {
                c.pair = c.res;
                p.elided = true;
                p.no_buffer = true;
                p.fused_into = i;
                if (p.src >= 0) net->layers[p.src].last_use = std::max(net->layers[p.src].last_use, i);   // read by layer i now
            }
        }

    // Concatenation in place: a convolution whose output is read by one concatenation only writes its channels
    // straight into that layer's buffer (row pitch = the joined channel count), so the join costs nothing.  Slices
    // start and end on 16-byte boundaries; anything else (pools, depthwise layers, shared producers, kept
    // activations) is copied into place when the concatenation layer runs.
    if (!net->training && !net->keep)
        for (int i = 0; i < n_layers; i++) {
            LayerPlan &cc = net->layers[i];
            if (cc.L.kind != SOL_LAYER_CONCAT || cc.out.c % 8 != 0) continue;
            const int owner = cc.chain_owner >= 0 ? cc.chain_owner : i;       // the layer whose buffer the parts are written into
            int off = 0, k = 0;
            for (int part : {cc.src, cc.res}) {
                LayerPlan &p = net->layers[part];
                if (k == 0 && p.L.kind == SOL_LAYER_CONCAT && p.chain_owner >= 0 && p.chain_owner == cc.chain_owner) {
                    cc.part_inplace[0] = true;                              // the chain's prefix: already there
                } else if (p.L.kind == SOL_LAYER_CONV && p.L.pool.kind == SOL_POOL_NONE && !p.absorbs_next && !p.elided && p.pair < 0 &&
                           p.nuse == 1 && p.out.c % 8 == 0 && off % 8 == 0) {
                    p.concat_into = owner;
                    p.concat_off = off;
                    cc.part_inplace[k] = true;
                }
                off += p.out.c;
                k++;
            }
        }

    // Depth-first bottleneck (the paper's layer-chain fusion, Sec. III-A, across three contractions): 1x1 reduce + ReLU,
    // 3x3 stride 1 + ReLU, 1x1 expand + identity shortcut + ReLU, every intermediate read by the next layer only, can run
    // as one launch that never stores the two intermediates (conv_block.hip).  The three layers keep their buffers, so
    // the plan can run them one by one as well: the shape heuristic below picks, sol_network_autotune measures.
    if (!net->training && !net->keep && dt == SOL_BF16)
        for (int i = 0; i < n_layers; i++) {
            LayerPlan &c3 = net->layers[i];
            const auto plain = [](const LayerPlan &l) {
                return l.L.kind == SOL_LAYER_CONV && l.L.pool.kind == SOL_POOL_NONE && l.L.act == SOL_ACT_RELU && !l.cout_real && !l.cin_real && !l.pre_bn && !l.ldx &&
                       l.concat_into < 0 && l.pair < 0 && !l.elided && !l.absorbs_next && l.cd.sh == 1 && l.cd.sw == 1;
            };
            const auto pointwise = [](const LayerPlan &l) { return l.cd.kh == 1 && l.cd.kw == 1 && l.cd.ph == 0 && l.cd.pw == 0; };
            if (!plain(c3) || !pointwise(c3) || c3.res < 0 || c3.src < 0) continue;
            LayerPlan &c2 = net->layers[c3.src];
            if (!plain(c2) || c2.res >= 0 || c2.nuse != 1 || c2.src < 0 || c2.cd.kh != 3 || c2.cd.kw != 3 || c2.cd.ph != 1 || c2.cd.pw != 1) continue;
            LayerPlan &c1 = net->layers[c2.src];
            if (!plain(c1) || !pointwise(c1) || c1.res >= 0 || c1.nuse != 1 || c1.src != c3.res || c1.src < 0) continue;
            if (c1.cd.cout != c2.cd.cout || c3.cd.cout != c1.cd.cin) continue;
            if (!block_kernel_applies(dt, c1.in.n, c1.in.h, c1.in.w, c1.in.c, c1.cd.cout)) continue;
            c3.block_c1 = c2.src; c3.block_c2 = c3.src;
            c1.block_c3 = c2.block_c3 = i;
            // heuristic: worth it where the pixels fill the chip several times over (the weights travel once per tile)
            c3.use_block = (long)c1.in.n * c1.in.h * c1.in.w >= 40000;
        }

    // Expand -> reduce pair (the same depth-first fusion across the border of two bottlenecks): the last 1x1 convolution of
    // a block (+ shortcut, ReLU) and the first 1x1 convolution of the next block, which reads nothing else, can run as
    // one launch that stores the block output once and never reads it back (conv_xr.hip).  Both layers keep their
    // buffers; a shape heuristic decides, sol_network_autotune measures.
    if (!net->training && !net->keep && dt == SOL_BF16)
        for (int i = 0; i + 1 < n_layers; i++) {
            LayerPlan &c3 = net->layers[i], &c1 = net->layers[i + 1];
            const auto plain1x1 = [](const LayerPlan &l) {
                return l.L.kind == SOL_LAYER_CONV && l.L.pool.kind == SOL_POOL_NONE && l.L.act == SOL_ACT_RELU && !l.cout_real && !l.cin_real && !l.pre_bn &&
                       !l.ldx && l.concat_into < 0 && l.pair < 0 && !l.elided && !l.absorbs_next && l.cd.sh == 1 && l.cd.sw == 1 && l.cd.kh == 1 &&
                       l.cd.kw == 1 && l.cd.ph == 0 && l.cd.pw == 0 && l.block_c1 < 0 && l.block_c3 < 0;
            };
            if (!plain1x1(c3) || !plain1x1(c1) || c3.res < 0 || c3.src < 0 || c1.src != i || c1.res >= 0 || c3.xr_from >= 0) continue;
            if (!xr_kernel_applies(dt, (long)c3.in.n * c3.in.h * c3.in.w, c3.cd.cin, c3.cd.cout, c1.cd.cout)) continue;
            c3.xr_next = i + 1;
            c1.xr_from = i;
            c3.use_xr = (long)c3.in.n * c3.in.h * c3.in.w >= 128 * 64;   // heuristic: a workgroup per 64 pixels; worth it once those fill half the chip
        }

    // activation layout: inference reuses buffers once their last consumer has run, training keeps all
    Arena ar;
    for (int i = 0; i < n_layers; i++) {
        LayerPlan &lp = net->layers[i];
        if (lp.split_pool) lp.tmp_off = ar.alloc(tensor_bytes(lp.conv_out));
        if (lp.chain_owner >= 0) {       // a join of a dense chain: a prefix of the chain's one buffer, laid out at the first touch
            LayerPlan &ow = net->layers[lp.chain_owner];
            if (!ow.prealloc) { ow.out_off = ar.alloc(tensor_bytes(ow.out)); ow.prealloc = true; }
            lp.out_off = ow.out_off;
        } else if (lp.absorbs_next) {   // writes the pool layer's output: that buffer has to exist while this layer runs
            if (i + 2 < n_layers) net->layers[i + 1].out_off = ar.alloc(tensor_bytes(net->layers[i + 1].out));
        } else if (lp.concat_into >= 0) {   // ... and so does the concatenation's, from its first in-place producer on
            LayerPlan &cc = net->layers[lp.concat_into];
            if (!cc.prealloc && lp.concat_into + 1 < n_layers) { cc.out_off = ar.alloc(tensor_bytes(cc.out)); cc.prealloc = true; }
        } else if (!lp.elided && !lp.prealloc && (i + 1 < n_layers || net->training)) {
            lp.out_off = ar.alloc(tensor_bytes(lp.out));
        }
        if (lp.xr_next >= 0 && lp.xr_next + 1 < n_layers) {   // this launch may also write the next layer's output: that buffer exists from here on
            LayerPlan &nx = net->layers[lp.xr_next];
            nx.out_off = ar.alloc(tensor_bytes(nx.out));
            nx.prealloc = true;
        }
        if (lp.split_pool && !net->keep) ar.release(lp.tmp_off);
        if (!net->keep)
            for (int j = 0; j < i; j++) {
                const LayerPlan &lj = net->layers[j];
                if (lj.last_use == i && j + 1 < n_layers && !lj.absorbs_next && lj.concat_into < 0 && !lj.no_buffer &&
                    !(lj.chain_owner >= 0 && lj.chain_owner != j))
                    ar.release(lj.out_off);
            }
    }
    if (net->training) SOL_TRY(plan_training(net, ar));
    net->ws_bytes = ar.top;
    return SOL_OK;
}

}  // namespace sol

using namespace sol;

extern "C" {

const char *sol_last_error(void) { return g_err; }
const char *sol_version(void) { return "libsol_mi355 0.1 (gfx950)"; }
int sol_out_size(int in, int k, int stride, int pad) { return out_size(in, k, stride, pad); }

// Debugging / sweeping aid: force the convolution tile for later calls of the calling thread (0 = automatic).
void sol_debug_set_conv_tile(int tile) { g_tile_override = tile; }

size_t sol_packed_weight_bytes(const sol_conv_desc *cd, sol_dtype dt) {
    if (!cd || cd->cout <= 0 || cd->cin <= 0 || cd->kh <= 0 || cd->kw <= 0) return 0;
    return (size_t)cd->cout * packed_k(*cd, dt) * dtype_size(dt);
}

sol_status sol_pack_conv_weights(const sol_conv_desc *cd, sol_dtype dt, const float *w_oihw, void *w_packed, void *stream) {
    SOL_TRY(check_conv(cd));
    SOL_REQUIRE(dt == SOL_F32 || dt == SOL_BF16, SOL_ERR_DTYPE, "unknown dtype %d", (int)dt);
    SOL_REQUIRE(w_oihw && w_packed, SOL_ERR_NULL, "weight pointers must not be NULL");
    SOL_REQUIRE(aligned16(w_oihw) && aligned16(w_packed), SOL_ERR_ALIGN, "device pointers must be 16-byte aligned");
    return launch_pack(*cd, dt, w_oihw, w_packed, false, (hipStream_t)stream);
}

sol_status sol_unpack_conv_weights(const sol_conv_desc *cd, sol_dtype dt, const void *w_packed, float *w_oihw, void *stream) {
    SOL_TRY(check_conv(cd));
    SOL_REQUIRE(dt == SOL_F32 || dt == SOL_BF16, SOL_ERR_DTYPE, "unknown dtype %d", (int)dt);
    SOL_REQUIRE(w_oihw && w_packed, SOL_ERR_NULL, "weight pointers must not be NULL");
    SOL_REQUIRE(aligned16(w_oihw) && aligned16(w_packed), SOL_ERR_ALIGN, "device pointers must be 16-byte aligned");
    return launch_pack(*cd, dt, w_oihw, const_cast<void *>(w_packed), true, (hipStream_t)stream);
}

sol_status sol_fold_bn(int c, const float *gamma, const float *beta, const float *mean, const float *var,
                       const float *bias, float eps, float *scale, float *shift, void *stream) {
    SOL_REQUIRE(c >= 0, SOL_ERR_SHAPE, "negative channel count %d", c);
    SOL_REQUIRE(scale && shift, SOL_ERR_NULL, "scale and shift must not be NULL");
    const bool any = gamma || beta || mean || var, all = gamma && beta && mean && var;
    SOL_REQUIRE(!any || all, SOL_ERR_NULL, "gamma, beta, mean, var must be all given or all NULL");
    SOL_REQUIRE(!any || eps >= 0.f, SOL_ERR_SHAPE, "negative eps");
    return launch_fold(c, gamma, beta, mean, var, bias, eps, scale, shift, (hipStream_t)stream);
}

sol_status sol_conv2d_fused(const sol_tensor_desc *xd, const void *x, const sol_conv_desc *cd, const void *w_packed,
                            const float *scale, const float *shift, const void *residual, int act,
                            const sol_pool_desc *pool, void *y, int32_t *pool_argmax, void *prepool, void *stream) {
    SOL_TRY(check_tensor(xd, "x"));
    SOL_TRY(check_conv(cd));
    return conv_fused_impl(*xd, x, *cd, w_packed, scale, shift, residual, act, pool, y, pool_argmax, prepool,
                           g_tile_override, (hipStream_t)stream);
}

sol_status sol_conv2d_preact_fused(const sol_tensor_desc *xd, const void *x, int ldx, const float *pre_scale, const float *pre_shift,
                                   const sol_conv_desc *cd, const void *w_packed, const float *scale, const float *shift,
                                   const void *residual, int act, const sol_pool_desc *pool, void *y, void *stream) {
    SOL_TRY(check_tensor(xd, "x"));
    SOL_TRY(check_conv(cd));
    SOL_REQUIRE(ldx >= 0, SOL_ERR_SHAPE, "negative input pitch");
    const InputSide ins{pre_scale, pre_shift, ldx, 0};
    return conv_fused_impl(*xd, x, *cd, w_packed, scale, shift, residual, act, pool, y, nullptr, nullptr, g_tile_override,
                           (hipStream_t)stream, 0, nullptr, &ins);
}

sol_status sol_bottleneck_fused(const sol_tensor_desc *xd, const void *x, int mid, const void *w1_packed, const float *scale1,
                                const float *shift1, const void *w2_packed, const float *scale2, const float *shift2,
                                const void *w3_packed, const float *scale3, const float *shift3, void *y, void *stream) {
    SOL_TRY(check_tensor(xd, "x"));
    SOL_REQUIRE(mid > 0, SOL_ERR_SHAPE, "bad mid channel count %d", mid);
    SOL_REQUIRE(block_kernel_applies(xd->dtype, xd->n, xd->h, xd->w, xd->c, mid), SOL_ERR_UNSUPPORTED,
                "the fused bottleneck runs bf16 blocks with 64 or 128 mid channels, a multiple of 128 block channels and images of at "
                "most %d columns (got dtype %d, %d mid channels, %d channels, %d columns); run the three layers one by one",
                mid == 64 ? 126 : 79, xd->dtype, mid, xd->c, xd->w);
    if (xd->n == 0) return SOL_OK;
    SOL_REQUIRE(x && y && w1_packed && w2_packed && w3_packed && scale1 && shift1 && scale2 && shift2 && scale3 && shift3, SOL_ERR_NULL,
                "x, y, the three packed weights and the six scale / shift vectors must not be NULL");
    SOL_REQUIRE(aligned16(x) && aligned16(y) && aligned16(w1_packed) && aligned16(w2_packed) && aligned16(w3_packed) && aligned16(scale1) &&
                    aligned16(shift1) && aligned16(scale2) && aligned16(shift2) && aligned16(scale3) && aligned16(shift3),
                SOL_ERR_ALIGN, "device pointers must be 16-byte aligned");
    SOL_REQUIRE(x != y, SOL_ERR_SHAPE, "the block cannot run in place: neighbouring tiles read x rows that others have already overwritten");
    const BlockLaunch b{x, y, w1_packed, w2_packed, w3_packed, scale1, shift1, scale2, shift2, scale3, shift3, xd->n, xd->h, xd->w, xd->c, mid};
    return launch_conv_block(b, (hipStream_t)stream);
}

sol_status sol_expand_reduce_fused(const sol_tensor_desc *td, const void *t, int c4, const void *w3_packed, const float *scale3, const float *shift3,
                                   const void *shortcut, void *y, int cz, const void *w1_packed, const float *scale1, const float *shift1, void *z,
                                   void *stream) {
    SOL_TRY(check_tensor(td, "t"));
    SOL_REQUIRE(td->dtype == SOL_BF16, SOL_ERR_DTYPE, "fused expand-reduce pair: bf16 only");
    SOL_REQUIRE(c4 > 0 && cz > 0, SOL_ERR_SHAPE, "bad channel counts %d, %d", c4, cz);
    const long P = (long)td->n * td->h * td->w;
    if (P == 0) return SOL_OK;
    SOL_REQUIRE(t && w3_packed && scale3 && shift3 && shortcut && y && w1_packed && scale1 && shift1 && z, SOL_ERR_NULL,
                "fused expand-reduce pair: every pointer is required");
    SOL_REQUIRE(aligned16(t) && aligned16(w3_packed) && aligned16(shortcut) && aligned16(y) && aligned16(w1_packed) && aligned16(z) &&
                    aligned16(scale3) && aligned16(shift3) && aligned16(scale1) && aligned16(shift1),
                SOL_ERR_ALIGN, "device pointers must be 16-byte aligned");
    SOL_REQUIRE(y != t && y != shortcut && z != t && z != y, SOL_ERR_UNSUPPORTED, "fused expand-reduce pair: outputs must not alias inputs");
    SOL_REQUIRE(xr_kernel_applies(td->dtype, P, td->c, c4, cz), SOL_ERR_UNSUPPORTED,
                "fused expand-reduce pair: needs 256 -> c4 -> 256 channels, c4 a multiple of 128 up to 1024");
    const XrLaunch xl{t, shortcut, y, z, w3_packed, w1_packed, scale3, shift3, scale1, shift1, P, td->c, c4, cz};
    return launch_conv_xr(xl, (hipStream_t)stream);
}

size_t sol_packed_dw_weight_bytes(int c, int kh, int kw, sol_dtype dt) {
    if (c <= 0 || kh <= 0 || kw <= 0) return 0;
    return dw_weight_bytes(c, kh, kw, dt);
}

sol_status sol_pack_dwconv_weights(int c, int kh, int kw, sol_dtype dt, const float *w_c1hw, void *w_packed, void *stream) {
    SOL_REQUIRE(c > 0 && kh > 0 && kw > 0 && (double)c * kh * kw < 1073741824.0, SOL_ERR_SHAPE, "bad depthwise weight shape c=%d k=%dx%d", c, kh, kw);
    SOL_REQUIRE(dt == SOL_F32 || dt == SOL_BF16, SOL_ERR_DTYPE, "unknown dtype %d", (int)dt);
    SOL_REQUIRE(w_c1hw && w_packed, SOL_ERR_NULL, "weight pointers must not be NULL");
    SOL_REQUIRE(aligned16(w_c1hw) && aligned16(w_packed), SOL_ERR_ALIGN, "device pointers must be 16-byte aligned");
    return launch_pack_dw(c, kh * kw, dt, w_c1hw, w_packed, (hipStream_t)stream);
}

sol_status sol_dwconv2d_fused(const sol_tensor_desc *xd, const void *x, const sol_conv_desc *cd, const void *w_packed,
                              const float *scale, const float *shift, const void *residual, int act, void *y, void *stream) {
    SOL_TRY(check_tensor(xd, "x"));
    SOL_TRY(check_conv(cd));
    return dwconv_impl(*xd, x, *cd, w_packed, scale, shift, residual, act, y, (hipStream_t)stream);
}

sol_status sol_linear(int m, int in_f, int out_f, sol_dtype dt, const void *x, const void *w_packed, const float *bias,
                      int act, void *y, void *stream) {
    SOL_REQUIRE(m >= 0 && in_f > 0 && out_f > 0, SOL_ERR_SHAPE, "bad linear shape m=%d in=%d out=%d", m, in_f, out_f);
    sol_tensor_desc xd{m, 1, 1, in_f, (int)dt};
    SOL_TRY(check_tensor(&xd, "x"));
    sol_conv_desc cd{out_f, in_f, 1, 1, 1, 1, 0, 0};
    return conv_fused_impl(xd, x, cd, w_packed, nullptr, bias, nullptr, act, nullptr, y, nullptr, nullptr,
                           g_tile_override, (hipStream_t)stream);
}

sol_status sol_pool(const sol_tensor_desc *xd, const void *x, const sol_pool_desc *pd, void *y, int32_t *argmax, void *stream) {
    SOL_TRY(check_tensor(xd, "x"));
    SOL_REQUIRE(pd, SOL_ERR_NULL, "pool descriptor is NULL");
    return pool_impl(*xd, x, *pd, y, argmax, (hipStream_t)stream);
}

sol_status sol_global_avgpool(const sol_tensor_desc *xd, const void *x, void *y, void *stream) {
    SOL_TRY(check_tensor(xd, "x"));
    if (xd->n == 0) return SOL_OK;
    SOL_REQUIRE(x && y, SOL_ERR_NULL, "x and y must not be NULL");
    SOL_REQUIRE(aligned16(x) && aligned16(y), SOL_ERR_ALIGN, "device pointers must be 16-byte aligned");
    return launch_gap(x, y, xd->n, xd->h * xd->w, xd->c, xd->dtype, (hipStream_t)stream);
}

// ---- network -----------------------------------------------------------------------------------------
static float *vec_ptr(const sol_network *net, const LayerPlan &lp, int which);

sol_status sol_network_create(const sol_layer *layers, int n_layers, const sol_tensor_desc *input, int flags,
                              sol_network **out) {
    const int training = flags & SOL_NET_TRAINING;
    SOL_REQUIRE(layers && out, SOL_ERR_NULL, "layers and out must not be NULL");
    SOL_REQUIRE(n_layers > 0, SOL_ERR_SHAPE, "empty layer list");
    SOL_TRY(check_tensor(input, "input"));
    sol_network *net = new (std::nothrow) sol_network();
    SOL_REQUIRE(net, SOL_ERR_HIP, "out of host memory");
    net->input = *input;
    net->training = training;
    net->keep = (flags & (SOL_NET_TRAINING | SOL_NET_KEEP_ACTIVATIONS)) != 0;
    net->params = nullptr;
    net->params_size = 0;
    sol_status s = plan_network(net, layers, n_layers);
    if (s != SOL_OK) { delete net; return s; }
    for (auto &lp : net->layers) lp.tile = lp.tile_dgrad = T_AUTO;
    *out = net;
    return SOL_OK;
}

void sol_network_destroy(sol_network *net) { delete net; }
size_t sol_network_param_bytes(const sol_network *net) { return net ? net->param_bytes : 0; }
size_t sol_network_workspace_bytes(const sol_network *net) { return net ? net->ws_bytes : 0; }
int sol_network_num_layers(const sol_network *net) { return net ? (int)net->layers.size() : 0; }

sol_status sol_network_output_desc(const sol_network *net, int layer, sol_tensor_desc *out) {
    SOL_REQUIRE(net && out, SOL_ERR_NULL, "net and out must not be NULL");
    if (layer == -1) layer = (int)net->layers.size() - 1;
    SOL_REQUIRE(layer >= 0 && layer < (int)net->layers.size(), SOL_ERR_SHAPE, "no layer %d", layer);
    *out = net->layers[layer].out;
    return SOL_OK;
}

sol_status sol_network_bind_params(sol_network *net, void *param_buf, size_t bytes) {
    SOL_REQUIRE(net, SOL_ERR_NULL, "net is NULL");
    SOL_REQUIRE(param_buf || net->param_bytes == 0, SOL_ERR_NULL, "param_buf is NULL");
    SOL_REQUIRE(bytes >= net->param_bytes, SOL_ERR_WORKSPACE, "parameter buffer has %zu bytes, %zu needed", bytes, net->param_bytes);
    SOL_REQUIRE(aligned16(param_buf), SOL_ERR_ALIGN, "parameter buffer must be 16-byte aligned");
    net->params = static_cast<unsigned char *>(param_buf);
    net->params_size = bytes;
    for (auto &lp : net->layers) lp.params_set = lp.pre_set = false;
    return SOL_OK;
}

sol_status sol_network_set_params(sol_network *net, int layer, const float *w, const float *gamma, const float *beta,
                                  const float *mean, const float *var, const float *bias, float eps, void *stream) {
    SOL_REQUIRE(net, SOL_ERR_NULL, "net is NULL");
    SOL_REQUIRE(layer >= 0 && layer < (int)net->layers.size(), SOL_ERR_SHAPE, "no layer %d", layer);
    LayerPlan &lp = net->layers[layer];
    const bool dwl = lp.L.kind == SOL_LAYER_DWCONV;
    SOL_REQUIRE(lp.L.kind == SOL_LAYER_CONV || lp.L.kind == SOL_LAYER_LINEAR || dwl, SOL_ERR_SHAPE, "layer %d has no parameters", layer);
    SOL_REQUIRE(net->params, SOL_ERR_WORKSPACE, "no parameter buffer bound (sol_network_bind_params)");
    SOL_REQUIRE(w, SOL_ERR_NULL, "w is NULL");
    const bool bn = (lp.L.kind == SOL_LAYER_CONV || dwl) && lp.L.has_bn;
    SOL_REQUIRE(!bn || (gamma && beta && (net->training || (mean && var))), SOL_ERR_NULL,
                "layer %d has batch-norm: gamma, beta%s required", layer, net->training ? "" : ", mean, var");
    SOL_REQUIRE(bn || !(gamma || beta || mean || var), SOL_ERR_SHAPE, "layer %d has no batch-norm", layer);
    SOL_REQUIRE(aligned16(w) && aligned16(gamma) && aligned16(beta) && aligned16(mean) && aligned16(var) && aligned16(bias),
                SOL_ERR_ALIGN, "device pointers must be 16-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    if (dwl)
        SOL_TRY(launch_pack_dw(lp.cd.cout, lp.cd.kh * lp.cd.kw, net->input.dtype, w, net->params + lp.w_off, st));
    else
        SOL_TRY(launch_pack(lp.cd, net->input.dtype, w, net->params + lp.w_off, false, st, lp.cout_real, lp.cin_real));
    if (net->training) {   // fp32 master copies, zero velocities, both packed orientations
        const size_t wn = (size_t)lp.cd.cout * lp.cd.cin * lp.cd.kh * lp.cd.kw * 4, cb = (size_t)lp.cd.cout * 4;
        SOL_HIP(hipMemcpyAsync(net->params + lp.master_off, w, wn, hipMemcpyDeviceToDevice, st));
        SOL_HIP(hipMemsetAsync(net->params + lp.vel_off, 0, wn, st));
        SOL_HIP(hipMemsetAsync(net->params + lp.vec_off, 0, VEC_COUNT * round_up(cb, 256), st));
        if (bn) {
            SOL_HIP(hipMemcpyAsync(vec_ptr(net, lp, VEC_GAMMA), gamma, cb, hipMemcpyDeviceToDevice, st));
            SOL_HIP(hipMemcpyAsync(vec_ptr(net, lp, VEC_BETA), beta, cb, hipMemcpyDeviceToDevice, st));
        }
        if (bias) SOL_HIP(hipMemcpyAsync(vec_ptr(net, lp, VEC_BIAS), bias, cb, hipMemcpyDeviceToDevice, st));
        if (lp.src >= 0) SOL_TRY(launch_pack_flip(lp.cd, net->input.dtype, w, net->params + lp.wT_off, st));
        lp.eps = eps;
        lp.params_set = true;
        return SOL_OK;
    }
    if (lp.cout_real) {     // padding channels: zero filters, shift 0 (scale irrelevant) -> they store 0 with or without ReLU
        SOL_HIP(hipMemsetAsync(net->params + lp.scale_off, 0, (size_t)lp.cd.cout * 4, st));
        SOL_HIP(hipMemsetAsync(net->params + lp.shift_off, 0, (size_t)lp.cd.cout * 4, st));
    }
    SOL_TRY(launch_fold(lp.cout_real ? lp.cout_real : lp.cd.cout, gamma, beta, mean, var, bias, eps,
                        reinterpret_cast<float *>(net->params + lp.scale_off), reinterpret_cast<float *>(net->params + lp.shift_off), st));
    lp.params_set = true;
    return SOL_OK;
}

sol_status sol_network_set_pre_bn(sol_network *net, int layer, const float *gamma, const float *beta, const float *mean, const float *var,
                                  float eps, void *stream) {
    SOL_REQUIRE(net, SOL_ERR_NULL, "net is NULL");
    SOL_REQUIRE(layer >= 0 && layer < (int)net->layers.size(), SOL_ERR_SHAPE, "no layer %d", layer);
    LayerPlan &lp = net->layers[layer];
    SOL_REQUIRE(lp.L.kind == SOL_LAYER_CONV && lp.pre_bn, SOL_ERR_SHAPE, "layer %d has no input-side batch-norm", layer);
    SOL_REQUIRE(net->params, SOL_ERR_WORKSPACE, "no parameter buffer bound (sol_network_bind_params)");
    SOL_REQUIRE(gamma && beta && mean && var, SOL_ERR_NULL, "gamma, beta, mean, var required");
    SOL_REQUIRE(aligned16(gamma) && aligned16(beta) && aligned16(mean) && aligned16(var), SOL_ERR_ALIGN, "device pointers must be 16-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    const int creal = lp.cin_real ? lp.cin_real : lp.cd.cin;
    float *ps = reinterpret_cast<float *>(net->params + lp.pre_scale_off), *ph = reinterpret_cast<float *>(net->params + lp.pre_shift_off);
    if (creal != lp.cd.cin) {      // channels beyond the real ones (reduction rounded up to whole chunks): constants 0, masked in the kernel anyway
        SOL_HIP(hipMemsetAsync(ps, 0, (size_t)lp.cd.cin * 4, st));
        SOL_HIP(hipMemsetAsync(ph, 0, (size_t)lp.cd.cin * 4, st));
    }
    SOL_TRY(launch_fold(creal, gamma, beta, mean, var, nullptr, eps, ps, ph, st));
    lp.pre_set = true;
    return SOL_OK;
}

static float *vec_ptr(const sol_network *net, const LayerPlan &lp, int which) {
    return reinterpret_cast<float *>(net->params + lp.vec_off + (size_t)which * round_up((size_t)lp.cd.cout * 4, 256));
}

static const void *layer_in(const sol_network *net, int idx, const void *x, const unsigned char *ws) {
    return idx < 0 ? x : static_cast<const void *>(ws + net->layers[idx].out_off);
}

// ---- training passes -----------------------------------------------------------------------------------
// The convolution launch of a training forward (BN layers store the bare convolution z) and of a training backward
// (data gradient into the producer's gradient buffer); shared by the passes and by the auto-tuner.
static sol_status train_conv_fwd(const sol_network *net, const LayerPlan &lp, const void *x, unsigned char *ws, int tile,
                                 hipStream_t st) {
    const void *in = layer_in(net, lp.src, x, ws);
    const bool bn = lp.L.kind == SOL_LAYER_CONV && lp.L.has_bn;
    const float *bias = vec_ptr(net, lp, VEC_BIAS);
    if (bn)
        return conv_fused_impl(lp.in, in, lp.cd, net->params + lp.w_off, nullptr, bias, nullptr, SOL_ACT_NONE, nullptr, ws + lp.z_off,
                               nullptr, nullptr, tile, st);
    const void *res = lp.res >= 0 ? layer_in(net, lp.res, x, ws) : nullptr;
    return conv_fused_impl(lp.in, in, lp.cd, net->params + lp.w_off, nullptr, bias, res, lp.L.act, nullptr, ws + lp.out_off, nullptr,
                           nullptr, tile, st);
}

static sol_status train_conv_dgrad(const sol_network *net, const LayerPlan &lp, const void *g, unsigned char *ws, int tile,
                                   hipStream_t st) {
    void *dsrc = ws + net->layers[lp.src].dact_off;
    return conv_fused_impl(lp.dzd, g, lp.dcd, net->params + lp.wT_off, nullptr, nullptr, lp.src_first ? nullptr : dsrc, SOL_ACT_NONE,
                           nullptr, dsrc, nullptr, nullptr, tile, st);
}

// Forward with batch statistics: conv -> z (stored), statistics of the stored z, then BN + residual + act
// in one elementwise pass.  Every output stays in the workspace for the backward pass.
static sol_status train_forward(sol_network *net, const void *x, void *y, unsigned char *ws, hipStream_t st) {
    const int nl = (int)net->layers.size(), dt = net->input.dtype;
    float *part = reinterpret_cast<float *>(ws + net->part_off);
    for (int i = 0; i < nl; i++) {
        const LayerPlan &lp = net->layers[i];
        const void *in = layer_in(net, lp.src, x, ws);
        void *out = ws + lp.out_off;
        switch (lp.L.kind) {
            case SOL_LAYER_CONV:
            case SOL_LAYER_LINEAR: {
                const bool bn = lp.L.kind == SOL_LAYER_CONV && lp.L.has_bn;
                const void *res = lp.res >= 0 ? layer_in(net, lp.res, x, ws) : nullptr;
                SOL_TRY(train_conv_fwd(net, lp, x, ws, g_tile_override ? g_tile_override : lp.tile, st));
                if (!bn) break;
                void *z = ws + lp.z_off;
                const int rows = lp.conv_out.n * lp.conv_out.h * lp.conv_out.w, C = lp.cd.cout;
                if (rows == 0) break;
                SOL_TRY(launch_bn_stats(z, rows, C, dt, lp.eps, vec_ptr(net, lp, VEC_MEAN), vec_ptr(net, lp, VEC_VAR),
                                        vec_ptr(net, lp, VEC_INVSTD), part, st));
                SOL_TRY(launch_bn_apply(z, res, out, vec_ptr(net, lp, VEC_MEAN), vec_ptr(net, lp, VEC_INVSTD),
                                        vec_ptr(net, lp, VEC_GAMMA), vec_ptr(net, lp, VEC_BETA), (long)rows * C, C,
                                        lp.L.act == SOL_ACT_RELU, dt, st));
                break;
            }
            case SOL_LAYER_POOL:
                SOL_TRY(pool_impl(lp.in, in, lp.L.pool, out,
                                  lp.L.pool.kind == SOL_POOL_MAX ? reinterpret_cast<int32_t *>(ws + lp.arg_off) : nullptr, st));
                break;
            case SOL_LAYER_GAP:
                if (lp.in.n > 0) SOL_TRY(launch_gap(in, out, lp.in.n, lp.in.h * lp.in.w, lp.in.c, lp.in.dtype, st));
                break;
        }
    }
    const LayerPlan &ll = net->layers[nl - 1];
    if (tensor_bytes(ll.out)) SOL_HIP(hipMemcpyAsync(y, ws + ll.out_off, tensor_bytes(ll.out), hipMemcpyDeviceToDevice, st));
    return SOL_OK;
}

static sol_status train_backward(sol_network *net, const void *x, const int32_t *labels, float *loss, unsigned char *ws,
                                 hipStream_t st) {
    const int nl = (int)net->layers.size(), dt = net->input.dtype;
    float *part = reinterpret_cast<float *>(ws + net->part_off);
    float *row_loss = reinterpret_cast<float *>(ws + net->loss_off);
    const LayerPlan &ll = net->layers[nl - 1];
    if (ll.out.n == 0) return SOL_OK;
    SOL_TRY(launch_softmax_ce(ws + ll.out_off, labels, ws + ll.dact_off, row_loss + 1, loss ? loss : row_loss, ll.out.n,
                              ll.out.c, dt, st));
    if (!net->side) {
        SOL_HIP(hipStreamCreateWithFlags(&net->side, hipStreamNonBlocking));
        SOL_HIP(hipEventCreateWithFlags(&net->ev_ready, hipEventDisableTiming));
        SOL_HIP(hipEventCreateWithFlags(&net->ev_join, hipEventDisableTiming));
    }
    hipStream_t side = net->side;
    bool side_busy = false;                 // the side stream holds work this call has not joined yet
    auto join_side = [&]() -> sol_status {  // `st` continues only after everything on the side stream
        if (side_busy) {
            SOL_HIP(hipEventRecord(net->ev_join, side));
            SOL_HIP(hipStreamWaitEvent(st, net->ev_join, 0));
            side_busy = false;
        }
        return SOL_OK;
    };
    struct PendingWgrad { const LayerPlan *lp; const void *in, *dz; };
    std::vector<PendingWgrad> pending;      // weight gradients whose dz is (or will be, in stream order) complete on `st`
    // every layer's weight-gradient partials stay in its own workspace region; one launch at the end adds them all
    WgradReduceBatch wred;
    wred.nseg = 0; wred.first_block[0] = 0;
    auto flush_wred = [&]() -> sol_status {
        SOL_TRY(join_side());
        const sol_status r = launch_wgrad_reduce_batch(wred, st);
        wred.nseg = 0; wred.first_block[0] = 0;
        return r;
    };
    auto flush_pending = [&]() -> sol_status {   // hand the collected weight gradients to the side stream
        if (pending.empty()) return SOL_OK;
        SOL_HIP(hipEventRecord(net->ev_ready, st));
        SOL_HIP(hipStreamWaitEvent(side, net->ev_ready, 0));
        for (const PendingWgrad &pw : pending) {
            const LayerPlan &lp = *pw.lp;
            int ns = 0;
            float *wpart = reinterpret_cast<float *>(ws + lp.wpart_off);
            float *dwp = reinterpret_cast<float *>(net->params + lp.grad_off);
            if (wred.nseg == WRED_MAX_SEG) SOL_TRY(flush_wred());
            SOL_TRY(launch_wgrad(lp.in, pw.in, lp.cd, pw.dz, lp.conv_out.h, lp.conv_out.w, dwp, wpart, side, &ns));
            side_busy = true;
            if (ns > 0) {
                const int j = wred.nseg++;
                wred.part[j] = wpart; wred.dw[j] = dwp; wred.nsplit[j] = ns;
                wred.K[j] = lp.cd.cout; wred.C[j] = lp.cd.cin; wred.RS[j] = lp.cd.kh * lp.cd.kw;
                wred.first_block[j + 1] = wred.first_block[j] + lp.cd.cout;
            }
        }
        pending.clear();
        return SOL_OK;
    };
    constexpr int kWgradGroup = 4;          // measured on the ResNet-18-shaped step: 1: 2.10, 2: 2.09, 4: 2.07, 8: 2.12 ms, all at the end: 2.27 ms
    for (int i = nl - 1; i >= 0; i--) {
        const LayerPlan &lp = net->layers[i];
        if (!lp.has_grad) continue;
        const void *in = layer_in(net, lp.src, x, ws);
        const void *dy = ws + lp.dact_off;
        void *dsrc = lp.src >= 0 ? static_cast<void *>(ws + net->layers[lp.src].dact_off) : nullptr;
        switch (lp.L.kind) {
            case SOL_LAYER_CONV:
            case SOL_LAYER_LINEAR: {
                const bool bn = lp.L.kind == SOL_LAYER_CONV && lp.L.has_bn;
                const int relu = lp.L.act == SOL_ACT_RELU;
                const int rows = lp.conv_out.n * lp.conv_out.h * lp.conv_out.w, C = lp.cd.cout;
                const long total = (long)rows * C;
                const void *yv = ws + lp.out_off;
                void *dres = lp.res >= 0 ? static_cast<void *>(ws + net->layers[lp.res].dact_off) : nullptr;
                unsigned char *dzbuf = ws + lp.dzl_off;
                const void *dz = dzbuf;
                if (bn) {
                    const void *z = ws + lp.z_off;
                    SOL_TRY(launch_grad_col_sums(z, dy, yv, vec_ptr(net, lp, VEC_MEAN), vec_ptr(net, lp, VEC_INVSTD), rows, C,
                                                 relu, dt, vec_ptr(net, lp, VEC_G_BETA), vec_ptr(net, lp, VEC_G_GAMMA), part, st));
                    SOL_TRY(launch_act_bn_bwd(z, dy, yv, vec_ptr(net, lp, VEC_MEAN), vec_ptr(net, lp, VEC_INVSTD),
                                              vec_ptr(net, lp, VEC_GAMMA), vec_ptr(net, lp, VEC_G_BETA),
                                              vec_ptr(net, lp, VEC_G_GAMMA), dzbuf, dres, lp.res_first, total, C, relu,
                                              1, rows, dt, st));
                } else {
                    if (relu || dres)
                        SOL_TRY(launch_act_bn_bwd(nullptr, dy, yv, nullptr, nullptr, nullptr, nullptr, nullptr, dzbuf,
                                                  dres, lp.res_first, total, C, relu, 0, rows, dt, st));
                    else
                        dz = dy;
                    SOL_TRY(launch_grad_col_sums(nullptr, dz, nullptr, nullptr, nullptr, rows, C, 0, dt,
                                                 vec_ptr(net, lp, VEC_G_BIAS), nullptr, part, st));
                }
                float *dwp = reinterpret_cast<float *>(net->params + lp.grad_off);
                if (rows > 0 && lp.cd.cin * lp.cd.kh * lp.cd.kw <= WRED_MAX_PLANE) {
                    pending.push_back(PendingWgrad{&lp, in, dz});
                    if ((int)pending.size() >= kWgradGroup) SOL_TRY(flush_pending());
                } else {
                    SOL_TRY(launch_wgrad(lp.in, in, lp.cd, dz, lp.conv_out.h, lp.conv_out.w, dwp, part, st));
                }
                if (lp.need_dgrad) {
                    const void *g = dz;
                    if (lp.dilate) {
                        SOL_TRY(launch_dilate(dz, ws + net->dil_off, lp.conv_out.n, lp.conv_out.h, lp.conv_out.w, C, lp.dzd.h,
                                              lp.dzd.w, lp.cd.sh, lp.cd.sw, dt, st));
                        g = ws + net->dil_off;
                    }
                    SOL_TRY(train_conv_dgrad(net, lp, g, ws, g_tile_override ? g_tile_override : lp.tile_dgrad, st));
                }
                break;
            }
            case SOL_LAYER_POOL: {
                if (!dsrc) break;
                PoolArgs a;
                const sol_pool_desc &pd = lp.L.pool;
                a.x = nullptr; a.y = nullptr; a.argmax = reinterpret_cast<int32_t *>(ws + lp.arg_off);
                a.N = lp.in.n; a.H = lp.in.h; a.W = lp.in.w; a.C = lp.in.c; a.Ho = lp.out.h; a.Wo = lp.out.w;
                a.kh = pd.kh; a.kw = pd.kw; a.sh = pd.sh; a.sw = pd.sw; a.ph = pd.ph; a.pw = pd.pw;
                a.kind = pd.kind; a.count_pad = pd.count_pad;
                SOL_TRY(launch_pool_bwd(a, dy, dsrc, lp.src_first, dt, st));
                break;
            }
            case SOL_LAYER_GAP:
                if (dsrc) SOL_TRY(launch_gap_bwd(dy, dsrc, lp.in.n, lp.in.h * lp.in.w, lp.in.c, lp.src_first, dt, st));
                break;
        }
    }
    SOL_TRY(flush_pending());
    return flush_wred();
}

static sol_status run_layers(sol_network *net, const void *x, void *y, void *workspace, size_t workspace_bytes,
                             int first, int last, hipStream_t st) {
    SOL_REQUIRE(net, SOL_ERR_NULL, "net is NULL");
    if (net->input.n == 0) return SOL_OK;                  // empty batch: every tensor is empty (allocators hand out NULL for them)
    SOL_REQUIRE(x && y, SOL_ERR_NULL, "x and y must not be NULL");
    SOL_REQUIRE(workspace || net->ws_bytes == 0, SOL_ERR_NULL, "workspace is NULL");
    SOL_REQUIRE(workspace_bytes >= net->ws_bytes, SOL_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, net->ws_bytes);
    SOL_REQUIRE(aligned16(x) && aligned16(y) && aligned16(workspace), SOL_ERR_ALIGN, "device pointers must be 16-byte aligned");
    const int nl = (int)net->layers.size();
    SOL_REQUIRE(first >= 0 && first <= last && last < nl, SOL_ERR_SHAPE, "bad layer range [%d,%d]", first, last);
    for (int i = first; i <= last; i++) {
        const LayerPlan &lp = net->layers[i];
        if (lp.L.kind == SOL_LAYER_CONV || lp.L.kind == SOL_LAYER_LINEAR || lp.L.kind == SOL_LAYER_DWCONV)
            SOL_REQUIRE(lp.params_set && (!lp.pre_bn || lp.pre_set), SOL_ERR_WORKSPACE, "layer %d: parameters not set", i);
    }
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    if (net->training) {
        SOL_REQUIRE(first == 0 && last == nl - 1, SOL_ERR_UNSUPPORTED, "training networks run whole passes only");
        return train_forward(net, x, y, ws, st);
    }
    for (int i = first; i <= last; i++) {
        const LayerPlan &lp = net->layers[i];
        if (lp.elided) continue;                            // computed by the convolution in front of it
        if (lp.block_c3 >= 0 && net->layers[lp.block_c3].use_block && !g_tile_override) continue;   // ... by the bottleneck launch behind it
        if (lp.xr_from >= 0 && net->layers[lp.xr_from].use_xr && !g_tile_override) continue;        // ... by the expand-reduce launch in front of it
        const void *in = layer_in(net, lp.src, x, ws);
        const int oi = lp.absorbs_next ? i + 1 : lp.concat_into >= 0 ? lp.concat_into : lp.chain_owner >= 0 ? lp.chain_owner : i;   // the layer whose buffer this launch writes
        void *out = oi + 1 == nl ? y : static_cast<void *>(ws + net->layers[oi].out_off);
        const size_t es = dtype_size(lp.in.dtype);
        int ldy = 0;
        if (lp.concat_into >= 0) {
            out = static_cast<unsigned char *>(out) + (size_t)lp.concat_off * es;
            ldy = net->layers[oi].out.c;
        }
        switch (lp.L.kind) {
            case SOL_LAYER_CONV: {
                const float *scale = reinterpret_cast<const float *>(net->params + lp.scale_off);
                const float *shift = reinterpret_cast<const float *>(net->params + lp.shift_off);
                const void *res = lp.res >= 0 ? layer_in(net, lp.res, x, ws) : nullptr;
                void *conv_dst = lp.split_pool ? static_cast<void *>(ws + lp.tmp_off) : out;
                const sol_pool_desc *fused = lp.absorbs_next ? &net->layers[i + 1].L.pool : lp.fuse_pool ? &lp.L.pool : nullptr;
                if (lp.block_c1 >= 0 && lp.use_block && !g_tile_override) {     // the whole bottleneck in one launch
                    const LayerPlan &b1 = net->layers[lp.block_c1], &b2 = net->layers[lp.block_c2];
                    const auto fp = [&](size_t off) { return reinterpret_cast<const float *>(net->params + off); };
                    const BlockLaunch bl{layer_in(net, b1.src, x, ws), conv_dst, net->params + b1.w_off, net->params + b2.w_off, net->params + lp.w_off,
                                         fp(b1.scale_off), fp(b1.shift_off), fp(b2.scale_off), fp(b2.shift_off), scale, shift,
                                         b1.in.n, b1.in.h, b1.in.w, b1.in.c, b1.cd.cout};
                    SOL_TRY(launch_conv_block(bl, st));
                    break;
                }
                if (lp.xr_next >= 0 && lp.use_xr && !g_tile_override) {        // this launch also computes the next bottleneck's first convolution
                    const LayerPlan &nx = net->layers[lp.xr_next];
                    const auto fp = [&](size_t off) { return reinterpret_cast<const float *>(net->params + off); };
                    void *z = lp.xr_next + 1 == nl ? y : static_cast<void *>(ws + nx.out_off);
                    const XrLaunch xl{in, res, conv_dst, z, net->params + lp.w_off, net->params + nx.w_off, scale, shift, fp(nx.scale_off), fp(nx.shift_off),
                                      (long)lp.in.n * lp.in.h * lp.in.w, lp.cd.cin, lp.cd.cout, nx.cd.cout};
                    SOL_TRY(launch_conv_xr(xl, st));
                    break;
                }
                if (lp.pair >= 0) {     // this launch also computes the projection shortcut it adds
                    const LayerPlan &pp = net->layers[lp.pair];
                    const PairOperand po{layer_in(net, pp.src, x, ws), net->params + pp.w_off,
                                         reinterpret_cast<const float *>(net->params + pp.scale_off),
                                         reinterpret_cast<const float *>(net->params + pp.shift_off),
                                         pp.in.h, pp.in.w, pp.cd.cin, packed_k(pp.cd, pp.in.dtype), pp.cd.sh};
                    SOL_TRY(conv_fused_impl(lp.in, in, lp.cd, net->params + lp.w_off, scale, shift, nullptr, lp.L.act, nullptr, conv_dst,
                                            nullptr, nullptr, T_AUTO, st, ldy, &po));
                    break;
                }
                if (lp.pre_bn || lp.ldx) {   // BN + ReLU on the input side and / or a channel prefix of a dense-block buffer
                    sol_tensor_desc xin = lp.in;
                    xin.c = lp.cd.cin;
                    const InputSide ins{lp.pre_bn ? reinterpret_cast<const float *>(net->params + lp.pre_scale_off) : nullptr,
                                        lp.pre_bn ? reinterpret_cast<const float *>(net->params + lp.pre_shift_off) : nullptr, lp.ldx,
                                        lp.ldx ? lp.cin_real : 0};
                    SOL_TRY(conv_fused_impl(xin, in, lp.cd, net->params + lp.w_off, scale, shift, res, lp.L.act, fused, conv_dst, nullptr,
                                            nullptr, g_tile_override ? g_tile_override : lp.tile, st, ldy, nullptr, &ins));
                    if (lp.split_pool) SOL_TRY(pool_impl(lp.conv_out, conv_dst, lp.L.pool, out, nullptr, st));
                    break;
                }
                SOL_TRY(conv_fused_impl(lp.in, in, lp.cd, net->params + lp.w_off, scale, shift, res, lp.L.act,
                                        fused, conv_dst, nullptr, nullptr,
                                        g_tile_override ? g_tile_override : lp.tile, st, ldy));
                if (lp.split_pool) SOL_TRY(pool_impl(lp.conv_out, conv_dst, lp.L.pool, out, nullptr, st));
                break;
            }
            case SOL_LAYER_LINEAR: {
                const float *shift = reinterpret_cast<const float *>(net->params + lp.shift_off);
                SOL_TRY(conv_fused_impl(lp.in, in, lp.cd, net->params + lp.w_off, nullptr, shift, nullptr, lp.L.act, nullptr,
                                        out, nullptr, nullptr, g_tile_override ? g_tile_override : lp.tile, st));
                break;
            }
            case SOL_LAYER_DWCONV: {
                const float *scale = reinterpret_cast<const float *>(net->params + lp.scale_off);
                const float *shift = reinterpret_cast<const float *>(net->params + lp.shift_off);
                const void *res = lp.res >= 0 ? layer_in(net, lp.res, x, ws) : nullptr;
                SOL_TRY(dwconv_impl(lp.in, in, lp.cd, net->params + lp.w_off, scale, shift, res, lp.L.act, out, st));
                break;
            }
            case SOL_LAYER_POOL: SOL_TRY(pool_impl(lp.in, in, lp.L.pool, out, nullptr, st)); break;
            case SOL_LAYER_GAP:
                if (lp.in.n > 0) SOL_TRY(launch_gap(in, out, lp.in.n, lp.in.h * lp.in.w, lp.in.c, lp.in.dtype, st));
                break;
            case SOL_LAYER_CONCAT: {    // only the parts their producers did not write in place
                int off = 0, k = 0;
                for (int part : {lp.src, lp.res}) {
                    const LayerPlan &p = net->layers[part];
                    if (!lp.part_inplace[k])
                        SOL_TRY(launch_concat_copy(layer_in(net, part, x, ws), out, (long)lp.out.n * lp.out.h * lp.out.w, p.out.c,
                                                   net->layers[oi].out.c, off, lp.out.dtype, st));
                    off += p.out.c;
                    k++;
                }
                break;
            }
        }
    }
    return SOL_OK;
}

sol_status sol_network_forward(sol_network *net, const void *x, void *y, void *workspace, size_t workspace_bytes, void *stream) {
    SOL_REQUIRE(net, SOL_ERR_NULL, "net is NULL");
    return run_layers(net, x, y, workspace, workspace_bytes, 0, (int)net->layers.size() - 1, (hipStream_t)stream);
}

// ---- forward pass with the activations in a static device array (allocates nothing, needs no caller workspace) ---------
// `scratch` below is a host-side stand-in for the device array: only the address hipGetSymbolAddress returns for
// the current device may be handed to kernels.  It is looked up once per device (every GPU holds its own copy of
// the array at its own address) and kept.
static __device__ __align__(256) unsigned char scratch[SOL_STATIC_WORKSPACE_BYTES];
static constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static unsigned char *g_scratch_ptr[kMaxDevices];      // per device, nullptr until that device's first call

static sol_status static_scratch(unsigned char **out) {
    int dev = -1;
    SOL_HIP(hipGetDevice(&dev));
    SOL_REQUIRE(dev >= 0 && dev < kMaxDevices, SOL_ERR_UNSUPPORTED, "device ordinal %d beyond the %d this library keeps scratch addresses for", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        SOL_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        SOL_REQUIRE(p && aligned16(p), SOL_ERR_HIP, "hipGetSymbolAddress returned %p for the static workspace", p);
        g_scratch_ptr[dev] = static_cast<unsigned char *>(p);
    }
    *out = g_scratch_ptr[dev];
    return SOL_OK;
}

sol_status sol_network_forward_static(sol_network *net, const void *x, void *y, void *stream) {
    SOL_REQUIRE(net, SOL_ERR_NULL, "net is NULL");
    SOL_REQUIRE(!net->training, SOL_ERR_UNSUPPORTED, "the static-workspace forward runs inference networks only (a backward pass needs the caller's workspace)");
    SOL_REQUIRE(net->ws_bytes <= (size_t)SOL_STATIC_WORKSPACE_BYTES, SOL_ERR_WORKSPACE,
                "network needs %zu bytes of workspace, the static workspace holds %zu (SOL_STATIC_WORKSPACE_BYTES); use sol_network_forward", net->ws_bytes,
                (size_t)SOL_STATIC_WORKSPACE_BYTES);
    unsigned char *ws = nullptr;
    SOL_TRY(static_scratch(&ws));
    return run_layers(net, x, y, ws, (size_t)SOL_STATIC_WORKSPACE_BYTES, 0, (int)net->layers.size() - 1, (hipStream_t)stream);
}

// ---- plan-time micro auto-tune ------------------------------------------------------------------------------
// Every kernel / tile id a convolution layer may be launched with (the launchers reject what does not fit a layer).
static const int kTuneCandidates[] = {
    T_256x128, T_128x128, T_128x64, T_256x64, T_64x64, T_128x32, T_128x256, T_64x128,
    D_128x128_64x4, D_128x128_64x3, D_256x128_64x3, D_128x64_64x4, D_64x64_64x4, D_128x256_64x3, D_256x64_64x3, D_64x128_64x4,
    D_128x128_128x2, D_128x128_128x3, D_128x64_128x3, D_64x64_128x3, D_128x128_64x5, D_64x64_128x4, D_256x128_128x3,
    D_256x128_64x4, D_128x256_64x4, D_64x64_64x8,
    H_256x128_x5, H_128x128_x3, H_256x64_x5, H_256x64_x6s, H_256x64_x6s2, H_256x64_x6, H_128x128_k2, H_64x128_k4, H_128x64_k4, H_64x64_k4,
    G_128x128_k2, G_256x128, G_128x256, G_64x128_k4, G_128x64_k4, G_256x256_r64, G_256x128_r64, G_64x64_k4, G_64x64_k4_deep};

// Training networks: the forward convolution of every layer and its data-gradient convolution get a tile each.
// A candidate is timed right behind another convolution of similar size that evicts its weights from L2 (the
// producer's forward convolution; for the data gradient the layer's own forward convolution), as it runs in a step.
// The timed launches overwrite activations and gradients: a forward pass must follow before the next backward.
static sol_status autotune_training(sol_network *net, const void *x, void *y, void *workspace, size_t workspace_bytes, int reps,
                                    hipStream_t st) {
    const int nl = (int)net->layers.size();
    for (auto &lp : net->layers) lp.tile = lp.tile_dgrad = T_AUTO;
    SOL_TRY(run_layers(net, x, y, workspace, workspace_bytes, 0, nl - 1, st));   // validates; fills every activation
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    SOL_HIP(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); SOL_FAIL(SOL_ERR_HIP, "hipEventCreate failed"); }
    sol_status rs = SOL_OK;
    // dg: time layer i's data gradient (else its forward convolution) with tile `tile`
    auto time_conv = [&](int i, bool dg, int tile, float *ms) -> sol_status {
        const LayerPlan &lp = net->layers[i];
        const int before = dg ? i : lp.src;
        const bool conv_before = before >= 0 && (net->layers[before].L.kind == SOL_LAYER_CONV);
        const void *g = ws + (lp.dilate ? net->dil_off : net->dz_off);
        float total = 0.f;
        for (int r = 0; r < reps + 1; r++) {
            if (conv_before) SOL_TRY(train_conv_fwd(net, net->layers[before], x, ws, net->layers[before].tile, st));
            SOL_HIP(hipEventRecord(e0, st));
            SOL_TRY(dg ? train_conv_dgrad(net, lp, g, ws, tile, st) : train_conv_fwd(net, lp, x, ws, tile, st));
            SOL_HIP(hipEventRecord(e1, st));
            SOL_HIP(hipEventSynchronize(e1));
            float t = 0.f;
            SOL_HIP(hipEventElapsedTime(&t, e0, e1));
            if (r > 0) total += t;
        }
        *ms = total;
        return SOL_OK;
    };
    // the gradient operands are whatever the workspace holds: make them finite numbers first
    if (net->dz_bytes) SOL_HIP(hipMemsetAsync(ws + net->dz_off, 0, net->dz_bytes, st));
    if (net->dil_bytes) SOL_HIP(hipMemsetAsync(ws + net->dil_off, 0, net->dil_bytes, st));
    for (int i = 0; i < nl && rs == SOL_OK; i++) {
        LayerPlan &lp = net->layers[i];
        if (lp.L.kind != SOL_LAYER_CONV || lp.in.n == 0) continue;
        for (int dg = 0; dg < 2 && rs == SOL_OK; dg++) {
            if (dg && !(lp.has_grad && lp.need_dgrad)) continue;
            float best = 0.f;
            rs = time_conv(i, dg, T_AUTO, &best);
            if (rs != SOL_OK) break;
            int best_tile = T_AUTO;
            for (int cand : kTuneCandidates) {
                float ms = 0.f;
                const sol_status cs = time_conv(i, dg, cand, &ms);
                if (cs == SOL_ERR_HIP) { rs = cs; break; }
                if (cs == SOL_OK && ms < 0.97f * best) { best = ms; best_tile = cand; }
            }
            (dg ? lp.tile_dgrad : lp.tile) = best_tile;
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rs != SOL_OK) for (auto &lp : net->layers) lp.tile = lp.tile_dgrad = T_AUTO;
    return rs;
}

sol_status sol_network_autotune(sol_network *net, const void *x, void *y, void *workspace, size_t workspace_bytes, int reps,
                                void *stream) {
    SOL_REQUIRE(net, SOL_ERR_NULL, "net is NULL");
    SOL_REQUIRE(reps >= 1 && reps <= 1000, SOL_ERR_SHAPE, "reps %d out of range [1,1000]", reps);
    if (net->training) return autotune_training(net, x, y, workspace, workspace_bytes, reps, (hipStream_t)stream);
    hipStream_t st = (hipStream_t)stream;
    const int nl = (int)net->layers.size();
    for (auto &lp : net->layers) { lp.tile = T_AUTO; lp.use_block = false; lp.use_xr = false; }   // every layer is tuned on its own first
    // one whole pass: validates the arguments and leaves finite activations of the right shape in every buffer
    SOL_TRY(run_layers(net, x, y, workspace, workspace_bytes, 0, nl - 1, st));
    hipEvent_t e0 = nullptr, e1 = nullptr;
    SOL_HIP(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); SOL_FAIL(SOL_ERR_HIP, "hipEventCreate failed"); }
    sol_status rs = SOL_OK;
    // Layer i timed the way it runs inside a pass: directly behind its producer, whose traffic leaves the layer's
    // input in the caches and pushes its weights out of L2 (a layer repeated back to back would find its weights
    // hot and favour the wrong kernels).  One event pair per launch, `reps` launches.
    auto time_layer = [&](int i, float *ms) -> sol_status {
        const int prod = net->layers[i].src >= 0 ? net->layers[i].src : -1;
        float total = 0.f;
        for (int r = 0; r < reps + 1; r++) {
            if (prod >= 0) SOL_TRY(run_layers(net, x, y, workspace, workspace_bytes, prod, prod, st));
            SOL_HIP(hipEventRecord(e0, st));
            SOL_TRY(run_layers(net, x, y, workspace, workspace_bytes, i, i, st));
            SOL_HIP(hipEventRecord(e1, st));
            SOL_HIP(hipEventSynchronize(e1));
            float t = 0.f;
            SOL_HIP(hipEventElapsedTime(&t, e0, e1));
            if (r > 0) total += t;                          // the first launch is a warm-up
        }
        *ms = total;
        return SOL_OK;
    };
    for (int i = 0; i < nl && rs == SOL_OK; i++) {
        LayerPlan &lp = net->layers[i];
        if (lp.L.kind != SOL_LAYER_CONV || lp.in.n == 0) continue;
        if (lp.absorbs_next || (lp.fuse_pool && !pool_is_fusable(lp.L.pool))) continue;   // stem + pool: one kernel, nothing to choose
        if (lp.elided || lp.pair >= 0) continue;                                          // projection pair: likewise
        float best = 0.f;
        rs = time_layer(i, &best);                            // the shape heuristic's choice is the incumbent
        if (rs != SOL_OK) break;
        int best_tile = T_AUTO;
        for (int cand : kTuneCandidates) {
            lp.tile = cand;
            float ms = 0.f;
            const sol_status cs = time_layer(i, &ms);
            if (cs == SOL_ERR_HIP) { rs = cs; break; }
            if (cs == SOL_OK && ms < 0.97f * best) { best = ms; best_tile = cand; }   // 3 % margin against timing noise
        }
        lp.tile = best_tile;
    }
    // bottlenecks: one depth-first launch against the three tuned launches, both right behind the block's producer
    for (int i = 0; i < nl && rs == SOL_OK; i++) {
        LayerPlan &lp = net->layers[i];
        if (lp.block_c1 < 0 || lp.in.n == 0) continue;
        const int c1 = lp.block_c1, c2 = lp.block_c2, prod = net->layers[c1].src;
        float t[2] = {0.f, 0.f};
        for (int fused = 0; fused < 2 && rs == SOL_OK; fused++) {
            lp.use_block = fused != 0;
            for (int r = 0; r < reps + 1 && rs == SOL_OK; r++) {
                if (prod >= 0) rs = run_layers(net, x, y, workspace, workspace_bytes, prod, prod, st);
                if (rs != SOL_OK) break;
                SOL_HIP(hipEventRecord(e0, st));
                for (int j : {c1, c2, i})
                    if (rs == SOL_OK) rs = run_layers(net, x, y, workspace, workspace_bytes, j, j, st);
                SOL_HIP(hipEventRecord(e1, st));
                SOL_HIP(hipEventSynchronize(e1));
                float ms = 0.f;
                SOL_HIP(hipEventElapsedTime(&ms, e0, e1));
                if (r > 0) t[fused] += ms;
            }
        }
        lp.use_block = t[1] < t[0];
    }
    // expand -> reduce pairs: one launch against the two tuned launches, both right behind the producer of the pair's input
    for (int i = 0; i < nl && rs == SOL_OK; i++) {
        LayerPlan &lp = net->layers[i];
        if (lp.xr_next < 0 || lp.in.n == 0) continue;
        const int prod = lp.src;
        float t[2] = {0.f, 0.f};
        for (int fused = 0; fused < 2 && rs == SOL_OK; fused++) {
            lp.use_xr = fused != 0;
            for (int r = 0; r < reps + 1 && rs == SOL_OK; r++) {
                if (prod >= 0) rs = run_layers(net, x, y, workspace, workspace_bytes, prod, prod, st);
                if (rs != SOL_OK) break;
                SOL_HIP(hipEventRecord(e0, st));
                for (int j : {i, lp.xr_next})
                    if (rs == SOL_OK) rs = run_layers(net, x, y, workspace, workspace_bytes, j, j, st);
                SOL_HIP(hipEventRecord(e1, st));
                SOL_HIP(hipEventSynchronize(e1));
                float ms = 0.f;
                SOL_HIP(hipEventElapsedTime(&ms, e0, e1));
                if (r > 0) t[fused] += ms;
            }
        }
        lp.use_xr = t[1] < t[0];
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rs != SOL_OK) for (auto &lp : net->layers) lp.tile = T_AUTO;
    return rs;
}

sol_status sol_network_layer_xr(const sol_network *net, int layer, int *state) {
    SOL_REQUIRE(net && state, SOL_ERR_NULL, "net and state must not be NULL");
    SOL_REQUIRE(layer >= 0 && layer < (int)net->layers.size(), SOL_ERR_SHAPE, "no layer %d", layer);
    const LayerPlan &lp = net->layers[layer];
    *state = lp.xr_next < 0 ? -1 : (lp.use_xr ? 1 : 0);
    return SOL_OK;
}

sol_status sol_network_set_layer_xr(sol_network *net, int layer, int fused) {
    SOL_REQUIRE(net, SOL_ERR_NULL, "net is NULL");
    SOL_REQUIRE(layer >= 0 && layer < (int)net->layers.size(), SOL_ERR_SHAPE, "no layer %d", layer);
    LayerPlan &lp = net->layers[layer];
    SOL_REQUIRE(lp.xr_next >= 0 || !fused, SOL_ERR_UNSUPPORTED, "layer %d is not the first layer of an expand-reduce pair the depth-first kernel can run", layer);
    lp.use_xr = fused != 0;
    return SOL_OK;
}

sol_status sol_network_layer_block(const sol_network *net, int layer, int *state) {
    SOL_REQUIRE(net && state, SOL_ERR_NULL, "net and state must not be NULL");
    SOL_REQUIRE(layer >= 0 && layer < (int)net->layers.size(), SOL_ERR_SHAPE, "no layer %d", layer);
    const LayerPlan &lp = net->layers[layer];
    *state = lp.block_c1 < 0 ? -1 : (lp.use_block ? 1 : 0);
    return SOL_OK;
}

sol_status sol_network_set_layer_block(sol_network *net, int layer, int fused) {
    SOL_REQUIRE(net, SOL_ERR_NULL, "net is NULL");
    SOL_REQUIRE(layer >= 0 && layer < (int)net->layers.size(), SOL_ERR_SHAPE, "no layer %d", layer);
    LayerPlan &lp = net->layers[layer];
    SOL_REQUIRE(lp.block_c1 >= 0 || !fused, SOL_ERR_UNSUPPORTED, "layer %d is not the last convolution of a bottleneck the depth-first kernel can run", layer);
    lp.use_block = fused != 0;
    return SOL_OK;
}

sol_status sol_network_set_layer_tile(sol_network *net, int layer, int tile) {
    SOL_REQUIRE(net, SOL_ERR_NULL, "net is NULL");
    SOL_REQUIRE(layer >= 0 && layer < (int)net->layers.size(), SOL_ERR_SHAPE, "no layer %d", layer);
    SOL_REQUIRE(tile >= 0 && tile < 100, SOL_ERR_SHAPE, "tile id %d out of range", tile);
    net->layers[layer].tile = tile;
    return SOL_OK;
}

sol_status sol_network_layer_tile(const sol_network *net, int layer, int *tile) {
    SOL_REQUIRE(net && tile, SOL_ERR_NULL, "net and tile must not be NULL");
    SOL_REQUIRE(layer >= 0 && layer < (int)net->layers.size(), SOL_ERR_SHAPE, "no layer %d", layer);
    *tile = net->layers[layer].tile;
    return SOL_OK;
}

// ---- HIP graph of one forward pass -------------------------------------------------------------------------
struct sol_graph {
    hipGraphExec_t exec;
};

sol_status sol_network_graph_create(sol_network *net, const void *x, void *y, void *workspace, size_t workspace_bytes,
                                    void *stream, sol_graph **out) {
    SOL_REQUIRE(net && out, SOL_ERR_NULL, "net and out must not be NULL");
    SOL_REQUIRE(!net->training, SOL_ERR_UNSUPPORTED, "graphs are recorded for inference networks only");
    SOL_REQUIRE(stream, SOL_ERR_UNSUPPORTED, "a graph cannot be recorded on the NULL stream");
    hipStream_t st = (hipStream_t)stream;
    const int last = (int)net->layers.size() - 1;
    // one eager pass first: validates the arguments and loads every kernel before the capture starts
    SOL_TRY(run_layers(net, x, y, workspace, workspace_bytes, 0, last, st));
    SOL_HIP(hipStreamSynchronize(st));
    SOL_HIP(hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal));
    const sol_status rs = run_layers(net, x, y, workspace, workspace_bytes, 0, last, st);
    hipGraph_t graph = nullptr;
    const hipError_t ce = hipStreamEndCapture(st, &graph);
    if (rs != SOL_OK) { if (graph) (void)hipGraphDestroy(graph); return rs; }
    SOL_REQUIRE(ce == hipSuccess && graph, SOL_ERR_HIP, "hipStreamEndCapture: %s", hipGetErrorString(ce));
    hipGraphExec_t exec = nullptr;
    const hipError_t ie = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    (void)hipGraphDestroy(graph);       // the executable graph holds what it needs
    SOL_REQUIRE(ie == hipSuccess && exec, SOL_ERR_HIP, "hipGraphInstantiate: %s", hipGetErrorString(ie));
    sol_graph *g = new (std::nothrow) sol_graph();
    if (!g) { (void)hipGraphExecDestroy(exec); SOL_FAIL(SOL_ERR_HIP, "out of host memory"); }
    g->exec = exec;
    *out = g;
    return SOL_OK;
}

sol_status sol_graph_launch(sol_graph *g, void *stream) {
    SOL_REQUIRE(g, SOL_ERR_NULL, "graph is NULL");
    SOL_HIP(hipGraphLaunch(g->exec, (hipStream_t)stream));
    return SOL_OK;
}

void sol_graph_destroy(sol_graph *g) {
    if (!g) return;
    (void)hipGraphExecDestroy(g->exec);
    delete g;
}

sol_status sol_network_layer_fused_into(const sol_network *net, int layer, int *into) {
    SOL_REQUIRE(net && into, SOL_ERR_NULL, "net / into is NULL");
    SOL_REQUIRE(layer >= 0 && layer < (int)net->layers.size(), SOL_ERR_SHAPE, "no layer %d", layer);
    const LayerPlan &lp = net->layers[layer];
    *into = (lp.block_c3 >= 0 && net->layers[lp.block_c3].use_block) ? lp.block_c3
            : (lp.xr_from >= 0 && net->layers[lp.xr_from].use_xr)        ? lp.xr_from
                                                                         : lp.fused_into;
    return SOL_OK;
}

sol_status sol_network_concat_in_place(const sol_network *net, int layer, int *parts) {
    SOL_REQUIRE(net && parts, SOL_ERR_NULL, "net / parts is NULL");
    SOL_REQUIRE(layer >= 0 && layer < (int)net->layers.size(), SOL_ERR_SHAPE, "no layer %d", layer);
    const LayerPlan &lp = net->layers[layer];
    SOL_REQUIRE(lp.L.kind == SOL_LAYER_CONCAT, SOL_ERR_SHAPE, "layer %d is not a concatenation", layer);
    *parts = (int)lp.part_inplace[0] + (int)lp.part_inplace[1];
    return SOL_OK;
}

sol_status sol_network_run_layer(sol_network *net, int layer, const void *x, void *y, void *workspace,
                                 size_t workspace_bytes, void *stream) {
    return run_layers(net, x, y, workspace, workspace_bytes, layer, layer, (hipStream_t)stream);
}

sol_status sol_network_layer_output(const sol_network *net, int layer, void *workspace, void **ptr) {
    SOL_REQUIRE(net && workspace && ptr, SOL_ERR_NULL, "net, workspace and ptr must not be NULL");
    SOL_REQUIRE(layer >= 0 && layer + (net->training ? 0 : 1) < (int)net->layers.size(), SOL_ERR_SHAPE,
                "layer %d has no workspace buffer (the last layer writes to y)", layer);
    *ptr = static_cast<unsigned char *>(workspace) + net->layers[layer].out_off;
    return SOL_OK;
}

sol_status sol_network_backward(sol_network *net, const void *x, const int32_t *labels, float *loss, void *workspace,
                                size_t workspace_bytes, void *stream) {
    SOL_REQUIRE(net, SOL_ERR_NULL, "net is NULL");
    SOL_REQUIRE(net->training, SOL_ERR_UNSUPPORTED, "network was not created with SOL_NET_TRAINING");
    SOL_REQUIRE(x && labels && workspace, SOL_ERR_NULL, "x, labels and workspace must not be NULL");
    SOL_REQUIRE(workspace_bytes >= net->ws_bytes, SOL_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, net->ws_bytes);
    SOL_REQUIRE(aligned16(x) && aligned16(workspace) && (reinterpret_cast<uintptr_t>(labels) & 3u) == 0 &&
                    (reinterpret_cast<uintptr_t>(loss) & 3u) == 0,
                SOL_ERR_ALIGN, "x and workspace must be 16-byte aligned, labels and loss 4-byte aligned");
    for (const auto &lp : net->layers)
        if (lp.L.kind == SOL_LAYER_CONV || lp.L.kind == SOL_LAYER_LINEAR)
            SOL_REQUIRE(lp.params_set, SOL_ERR_WORKSPACE, "parameters not set");
    return train_backward(net, x, labels, loss, static_cast<unsigned char *>(workspace), (hipStream_t)stream);
}

sol_status sol_network_sgd_step(sol_network *net, float lr, float momentum, void *stream) {
    SOL_REQUIRE(net, SOL_ERR_NULL, "net is NULL");
    SOL_REQUIRE(net->training, SOL_ERR_UNSUPPORTED, "network was not created with SOL_NET_TRAINING");
    SOL_REQUIRE(net->params, SOL_ERR_WORKSPACE, "no parameter buffer bound (sol_network_bind_params)");
    hipStream_t st = (hipStream_t)stream;
    // every tensor update in one launch, every re-pack in a second one (the tables travel in the kernel arguments;
    // networks with more tensors than a table holds take several launches)
    SgdBatch sb;
    PackBatch pb;
    sb.nseg = 0; sb.first_block[0] = 0;
    pb.nseg = 0; pb.first_block[0] = 0;
    auto flush_sgd = [&]() -> sol_status {
        const sol_status r = launch_sgd_batch(sb, lr, momentum, st);
        sb.nseg = 0; sb.first_block[0] = 0;
        return r;
    };
    auto flush_pack = [&]() -> sol_status {
        const sol_status r = launch_pack_batch(pb, net->input.dtype, st);
        pb.nseg = 0; pb.first_block[0] = 0;
        return r;
    };
    auto add_sgd = [&](float *w, float *v, const float *g, long n) -> sol_status {
        if (n <= 0) return SOL_OK;
        if (sb.nseg == SGD_MAX_SEG) SOL_TRY(flush_sgd());
        const int i = sb.nseg++;
        sb.w[i] = w; sb.v[i] = v; sb.g[i] = g; sb.n[i] = n;
        sb.first_block[i + 1] = sb.first_block[i] + (int)((n + SGD_ELEMS_PER_BLOCK - 1) / SGD_ELEMS_PER_BLOCK);
        return SOL_OK;
    };
    auto add_pack = [&](const float *w, void *out, const sol_conv_desc &cd, bool flip) -> sol_status {
        const sol_conv_desc td{cd.cin, cd.cout, cd.kh, cd.kw, 1, 1, 0, 0};   // the flipped pack belongs to the transposed convolution
        const int Kp = packed_k(flip ? td : cd, net->input.dtype);
        const long total = (long)(flip ? cd.cin : cd.cout) * Kp;
        if (total <= 0) return SOL_OK;
        if (pb.nseg == PACK_MAX_SEG) SOL_TRY(flush_pack());
        const int i = pb.nseg++;
        pb.w[i] = w; pb.out[i] = out; pb.K[i] = cd.cout; pb.C[i] = cd.cin; pb.R[i] = cd.kh; pb.S[i] = cd.kw; pb.Kp[i] = Kp;
        pb.flip[i] = flip ? 1 : 0;
        pb.first_block[i + 1] = pb.first_block[i] + pack_segment_blocks(cd.cout, cd.cin, cd.kh, cd.kw, Kp, pb.flip[i], &pb.mode[i]);
        return SOL_OK;
    };
    for (const auto &lp : net->layers) {
        if (!(lp.L.kind == SOL_LAYER_CONV || lp.L.kind == SOL_LAYER_LINEAR) || !lp.has_grad) continue;
        SOL_REQUIRE(lp.params_set, SOL_ERR_WORKSPACE, "parameters not set");
        const bool bn = lp.L.kind == SOL_LAYER_CONV && lp.L.has_bn;
        float *w = reinterpret_cast<float *>(net->params + lp.master_off);
        SOL_TRY(add_sgd(w, reinterpret_cast<float *>(net->params + lp.vel_off), reinterpret_cast<const float *>(net->params + lp.grad_off),
                        (long)lp.cd.cout * lp.cd.cin * lp.cd.kh * lp.cd.kw));
        if (bn) {
            SOL_TRY(add_sgd(vec_ptr(net, lp, VEC_GAMMA), vec_ptr(net, lp, VEC_V_GAMMA), vec_ptr(net, lp, VEC_G_GAMMA), lp.cd.cout));
            SOL_TRY(add_sgd(vec_ptr(net, lp, VEC_BETA), vec_ptr(net, lp, VEC_V_BETA), vec_ptr(net, lp, VEC_G_BETA), lp.cd.cout));
        } else {
            SOL_TRY(add_sgd(vec_ptr(net, lp, VEC_BIAS), vec_ptr(net, lp, VEC_V_BIAS), vec_ptr(net, lp, VEC_G_BIAS), lp.cd.cout));
        }
    }
    SOL_TRY(flush_sgd());
    for (const auto &lp : net->layers) {           // behind the update on the same stream
        if (!(lp.L.kind == SOL_LAYER_CONV || lp.L.kind == SOL_LAYER_LINEAR) || !lp.has_grad) continue;
        const float *w = reinterpret_cast<const float *>(net->params + lp.master_off);
        SOL_TRY(add_pack(w, net->params + lp.w_off, lp.cd, false));
        if (lp.src >= 0) SOL_TRY(add_pack(w, net->params + lp.wT_off, lp.cd, true));
    }
    SOL_TRY(flush_pack());
    return SOL_OK;
}

sol_status sol_network_tensor(const sol_network *net, int layer, int which, float **ptr, size_t *count) {
    SOL_REQUIRE(net && ptr && count, SOL_ERR_NULL, "net, ptr and count must not be NULL");
    SOL_REQUIRE(net->training, SOL_ERR_UNSUPPORTED, "network was not created with SOL_NET_TRAINING");
    SOL_REQUIRE(net->params, SOL_ERR_WORKSPACE, "no parameter buffer bound (sol_network_bind_params)");
    SOL_REQUIRE(layer >= 0 && layer < (int)net->layers.size(), SOL_ERR_SHAPE, "no layer %d", layer);
    const LayerPlan &lp = net->layers[layer];
    SOL_REQUIRE(lp.L.kind == SOL_LAYER_CONV || lp.L.kind == SOL_LAYER_LINEAR, SOL_ERR_SHAPE, "layer %d has no parameters", layer);
    const size_t wn = (size_t)lp.cd.cout * lp.cd.cin * lp.cd.kh * lp.cd.kw;
    switch (which) {
        case SOL_NT_W: *ptr = reinterpret_cast<float *>(net->params + lp.master_off); *count = wn; break;
        case SOL_NT_GRAD_W: *ptr = reinterpret_cast<float *>(net->params + lp.grad_off); *count = wn; break;
        case SOL_NT_GAMMA: *ptr = vec_ptr(net, lp, VEC_GAMMA); *count = lp.cd.cout; break;
        case SOL_NT_BETA: *ptr = vec_ptr(net, lp, VEC_BETA); *count = lp.cd.cout; break;
        case SOL_NT_BIAS: *ptr = vec_ptr(net, lp, VEC_BIAS); *count = lp.cd.cout; break;
        case SOL_NT_GRAD_GAMMA: *ptr = vec_ptr(net, lp, VEC_G_GAMMA); *count = lp.cd.cout; break;
        case SOL_NT_GRAD_BETA: *ptr = vec_ptr(net, lp, VEC_G_BETA); *count = lp.cd.cout; break;
        case SOL_NT_GRAD_BIAS: *ptr = vec_ptr(net, lp, VEC_G_BIAS); *count = lp.cd.cout; break;
        case SOL_NT_MEAN: *ptr = vec_ptr(net, lp, VEC_MEAN); *count = lp.cd.cout; break;
        case SOL_NT_VAR: *ptr = vec_ptr(net, lp, VEC_VAR); *count = lp.cd.cout; break;
        case SOL_NT_VEL_W: *ptr = reinterpret_cast<float *>(net->params + lp.vel_off); *count = wn; break;
        case SOL_NT_VEL_GAMMA: *ptr = vec_ptr(net, lp, VEC_V_GAMMA); *count = lp.cd.cout; break;
        case SOL_NT_VEL_BETA: *ptr = vec_ptr(net, lp, VEC_V_BETA); *count = lp.cd.cout; break;
        case SOL_NT_VEL_BIAS: *ptr = vec_ptr(net, lp, VEC_V_BIAS); *count = lp.cd.cout; break;
        default: SOL_FAIL(SOL_ERR_SHAPE, "unknown tensor id %d", which);
    }
    return SOL_OK;
}

sol_status sol_network_layer_preact(const sol_network *net, int layer, void *workspace, void **ptr) {
    SOL_REQUIRE(net && workspace && ptr, SOL_ERR_NULL, "net, workspace and ptr must not be NULL");
    SOL_REQUIRE(net->training, SOL_ERR_UNSUPPORTED, "network was not created with SOL_NET_TRAINING");
    SOL_REQUIRE(layer >= 0 && layer < (int)net->layers.size(), SOL_ERR_SHAPE, "no layer %d", layer);
    const LayerPlan &lp = net->layers[layer];
    SOL_REQUIRE(lp.L.kind == SOL_LAYER_CONV && lp.L.has_bn, SOL_ERR_SHAPE, "layer %d is not a convolution with BN", layer);
    *ptr = static_cast<unsigned char *>(workspace) + lp.z_off;
    return SOL_OK;
}

sol_status sol_network_layer_grad(const sol_network *net, int layer, void *workspace, void **ptr) {
    SOL_REQUIRE(net && workspace && ptr, SOL_ERR_NULL, "net, workspace and ptr must not be NULL");
    SOL_REQUIRE(net->training, SOL_ERR_UNSUPPORTED, "network was not created with SOL_NET_TRAINING");
    SOL_REQUIRE(layer >= 0 && layer < (int)net->layers.size(), SOL_ERR_SHAPE, "no layer %d", layer);
    SOL_REQUIRE(net->layers[layer].has_grad, SOL_ERR_SHAPE, "layer %d receives no gradient", layer);
    *ptr = static_cast<unsigned char *>(workspace) + net->layers[layer].dact_off;
    return SOL_OK;
}

}  // extern "C"

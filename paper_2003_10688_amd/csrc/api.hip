// C ABI of the library: argument validation, the single fused-layer entry points, and the network
// object (planner + executor).  Host code only; all device work is in conv_igemm.hip / fusion.hip.
#include <stdarg.h>

#include <algorithm>
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

static int g_tile_override = 0;   // debugging / sweeping aid, see sol_debug_set_conv_tile

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

// Shared by sol_conv2d_fused and the network executor.
static sol_status conv_fused_impl(const sol_tensor_desc &xd, const void *x, const sol_conv_desc &cd, const void *w,
                                  const float *scale, const float *shift, const void *res, int act,
                                  const sol_pool_desc *pool, void *y, int32_t *argmax, void *prepool, int tile,
                                  hipStream_t st) {
    SOL_REQUIRE(cd.cin == xd.c, SOL_ERR_SHAPE, "conv cin %d != input channels %d", cd.cin, xd.c);
    SOL_REQUIRE(act == SOL_ACT_NONE || act == SOL_ACT_RELU, SOL_ERR_SHAPE, "bad activation %d", act);
    const int Ho = out_size(xd.h, cd.kh, cd.sh, cd.ph), Wo = out_size(xd.w, cd.kw, cd.sw, cd.pw);
    SOL_REQUIRE(xd.h + 2 * cd.ph >= cd.kh && xd.w + 2 * cd.pw >= cd.kw && Ho > 0 && Wo > 0, SOL_ERR_SHAPE,
                "filter %dx%d larger than padded input %dx%d", cd.kh, cd.kw, xd.h + 2 * cd.ph, xd.w + 2 * cd.pw);
    ConvArgs a;
    memset(static_cast<void *>(&a), 0, sizeof(a));
    a.pool = 0;
    a.Hy = Ho; a.Wy = Wo;
    if (pool && pool->kind != SOL_POOL_NONE) {
        SOL_TRY(check_pool(pool));
        SOL_REQUIRE(pool_is_fusable(*pool), SOL_ERR_UNSUPPORTED,
                    "only a 2x2 stride-2 unpadded pool can be fused into the convolution; run sol_pool separately");
        a.pool = pool->kind == SOL_POOL_MAX ? 1 : 2;
        a.Hy = Ho / 2; a.Wy = Wo / 2;
        SOL_REQUIRE(a.Hy > 0 && a.Wy > 0, SOL_ERR_SHAPE, "conv output %dx%d too small for a 2x2 pool", Ho, Wo);
    }
    SOL_REQUIRE((double)xd.n * Ho * Wo * cd.cout < 2147483648.0, SOL_ERR_UNSUPPORTED, "output has 2^31 elements or more");
    if (xd.n == 0) return SOL_OK;
    SOL_REQUIRE(x && w && y, SOL_ERR_NULL, "x, w_packed and y must not be NULL");
    SOL_REQUIRE(aligned16(x) && aligned16(w) && aligned16(y) && aligned16(scale) && aligned16(shift) && aligned16(res) &&
                    aligned16(argmax) && aligned16(prepool),
                SOL_ERR_ALIGN, "device pointers must be 16-byte aligned");
    a.x = x; a.w = w; a.scale = scale; a.shift = shift; a.res = res; a.y = y;
    a.argmax = a.pool == 1 ? argmax : nullptr;
    a.prepool = a.pool ? prepool : nullptr;
#ifdef SOL_PHASE_TIMING
    a.prepool = prepool;   // profiling build: receives per-phase cycle counts
#endif
    a.N = xd.n; a.H = xd.h; a.W = xd.w; a.C = xd.c;
    a.Cout = cd.cout; a.R = cd.kh; a.S = cd.kw; a.sh = cd.sh; a.sw = cd.sw; a.ph = cd.ph; a.pw = cd.pw;
    a.Ho = Ho; a.Wo = Wo;
    a.P = a.pool ? xd.n * a.Hy * a.Wy * 4 : xd.n * Ho * Wo;
    a.Kp = packed_k(cd, xd.dtype);
    a.Ktot = cd.kh * cd.kw * cd.cin;
    a.act = act;
    a.dw = FastDiv((uint32_t)(a.pool ? a.Wy : Wo));
    a.dh = FastDiv((uint32_t)(a.pool ? a.Hy : Ho));
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

// ---- network ---------------------------------------------------------------------------------------
struct LayerPlan {
    sol_layer L;
    sol_tensor_desc in, out;        // input / stored output
    sol_tensor_desc conv_out;       // CONV: convolution output (before any pool)
    sol_conv_desc cd;               // CONV / LINEAR (as 1x1)
    int src, res;                   // resolved producer indices, -1 = network input
    bool fuse_pool, split_pool;     // CONV with pool: fused into the epilogue, or run as a second launch
    size_t w_off, scale_off, shift_off;
    size_t out_off, tmp_off;        // workspace offsets; out_off unused for the last layer
    int last_use;
    bool params_set;
};

}  // namespace sol

struct sol_network {
    std::vector<sol::LayerPlan> layers;
    sol_tensor_desc input;
    int training, keep;
    size_t param_bytes, ws_bytes;
    unsigned char *params;
    size_t params_size;
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

static sol_status plan_network(sol_network *net, const sol_layer *layers, int n_layers) {
    const int dt = net->input.dtype;
    net->layers.resize(n_layers);
    size_t poff = 0;
    for (int i = 0; i < n_layers; i++) {
        LayerPlan &lp = net->layers[i];
        memset(&lp, 0, sizeof(lp));
        lp.L = layers[i];
        const sol_layer &L = lp.L;
        SOL_REQUIRE(L.src >= -1 && L.src < i, SOL_ERR_SHAPE, "layer %d: src %d must name an earlier layer", i, L.src);
        lp.src = L.src == -1 ? i - 1 : L.src;
        lp.res = -1;
        lp.in = lp.src < 0 ? net->input : net->layers[lp.src].out;
        lp.out = lp.in;
        lp.last_use = i;
        switch (L.kind) {
            case SOL_LAYER_CONV: {
                lp.cd = L.conv;
                lp.cd.cin = lp.in.c;
                SOL_TRY(check_conv(&lp.cd));
                SOL_REQUIRE(lp.in.h + 2 * lp.cd.ph >= lp.cd.kh && lp.in.w + 2 * lp.cd.pw >= lp.cd.kw, SOL_ERR_SHAPE,
                            "layer %d: filter larger than padded input", i);
                lp.conv_out = lp.in;
                lp.conv_out.h = out_size(lp.in.h, lp.cd.kh, lp.cd.sh, lp.cd.ph);
                lp.conv_out.w = out_size(lp.in.w, lp.cd.kw, lp.cd.sw, lp.cd.pw);
                lp.conv_out.c = lp.cd.cout;
                lp.out = lp.conv_out;
                if (L.pool.kind != SOL_POOL_NONE) {
                    SOL_TRY(check_pool(&L.pool));
                    lp.fuse_pool = pool_is_fusable(L.pool);
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
        if (L.kind == SOL_LAYER_CONV || L.kind == SOL_LAYER_LINEAR) {
            lp.w_off = poff; poff += round_up(sol_packed_weight_bytes(&lp.cd, (sol_dtype)dt), 256);
            lp.scale_off = poff; poff += round_up((size_t)lp.cd.cout * 4, 256);
            lp.shift_off = poff; poff += round_up((size_t)lp.cd.cout * 4, 256);
        }
        if (lp.src >= 0) net->layers[lp.src].last_use = i;
        if (lp.res >= 0) net->layers[lp.res].last_use = std::max(net->layers[lp.res].last_use, i);
    }
    net->param_bytes = poff;

    // activation layout: inference reuses buffers once their last consumer has run, training keeps all
    Arena ar;
    for (int i = 0; i < n_layers; i++) {
        LayerPlan &lp = net->layers[i];
        if (lp.split_pool) lp.tmp_off = ar.alloc(tensor_bytes(lp.conv_out));
        if (i + 1 < n_layers) lp.out_off = ar.alloc(tensor_bytes(lp.out));
        if (lp.split_pool && !net->keep) ar.release(lp.tmp_off);
        if (!net->keep)
            for (int j = 0; j < i; j++)
                if (net->layers[j].last_use == i && j + 1 < n_layers) ar.release(net->layers[j].out_off);
    }
    net->ws_bytes = ar.top;
    return SOL_OK;
}

}  // namespace sol

using namespace sol;

extern "C" {

const char *sol_last_error(void) { return g_err; }
const char *sol_version(void) { return "libsol_mi355 0.1 (gfx950)"; }
int sol_out_size(int in, int k, int stride, int pad) { return out_size(in, k, stride, pad); }

// Debugging / sweeping aid: force the convolution tile (0 = automatic).  Not part of the stable ABI.
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
sol_status sol_network_create(const sol_layer *layers, int n_layers, const sol_tensor_desc *input, int flags,
                              sol_network **out) {
    const int training = flags & SOL_NET_TRAINING;
    SOL_REQUIRE(layers && out, SOL_ERR_NULL, "layers and out must not be NULL");
    SOL_REQUIRE(n_layers > 0, SOL_ERR_SHAPE, "empty layer list");
    SOL_TRY(check_tensor(input, "input"));
    SOL_REQUIRE(!training, SOL_ERR_UNSUPPORTED, "training networks are not available in this build");
    sol_network *net = new (std::nothrow) sol_network();
    SOL_REQUIRE(net, SOL_ERR_HIP, "out of host memory");
    net->input = *input;
    net->training = training;
    net->keep = (flags & (SOL_NET_TRAINING | SOL_NET_KEEP_ACTIVATIONS)) != 0;
    net->params = nullptr;
    net->params_size = 0;
    sol_status s = plan_network(net, layers, n_layers);
    if (s != SOL_OK) { delete net; return s; }
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
    for (auto &lp : net->layers) lp.params_set = false;
    return SOL_OK;
}

sol_status sol_network_set_params(sol_network *net, int layer, const float *w, const float *gamma, const float *beta,
                                  const float *mean, const float *var, const float *bias, float eps, void *stream) {
    SOL_REQUIRE(net, SOL_ERR_NULL, "net is NULL");
    SOL_REQUIRE(layer >= 0 && layer < (int)net->layers.size(), SOL_ERR_SHAPE, "no layer %d", layer);
    LayerPlan &lp = net->layers[layer];
    SOL_REQUIRE(lp.L.kind == SOL_LAYER_CONV || lp.L.kind == SOL_LAYER_LINEAR, SOL_ERR_SHAPE, "layer %d has no parameters", layer);
    SOL_REQUIRE(net->params, SOL_ERR_WORKSPACE, "no parameter buffer bound (sol_network_bind_params)");
    SOL_REQUIRE(w, SOL_ERR_NULL, "w is NULL");
    const bool bn = lp.L.kind == SOL_LAYER_CONV && lp.L.has_bn;
    SOL_REQUIRE(!bn || (gamma && beta && mean && var), SOL_ERR_NULL, "layer %d has batch-norm: gamma, beta, mean, var required", layer);
    SOL_REQUIRE(bn || !(gamma || beta || mean || var), SOL_ERR_SHAPE, "layer %d has no batch-norm", layer);
    SOL_REQUIRE(aligned16(w) && aligned16(gamma) && aligned16(beta) && aligned16(mean) && aligned16(var) && aligned16(bias),
                SOL_ERR_ALIGN, "device pointers must be 16-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    SOL_TRY(launch_pack(lp.cd, net->input.dtype, w, net->params + lp.w_off, false, st));
    SOL_TRY(launch_fold(lp.cd.cout, gamma, beta, mean, var, bias, eps, reinterpret_cast<float *>(net->params + lp.scale_off),
                        reinterpret_cast<float *>(net->params + lp.shift_off), st));
    lp.params_set = true;
    return SOL_OK;
}

static const void *layer_in(const sol_network *net, int idx, const void *x, const unsigned char *ws) {
    return idx < 0 ? x : static_cast<const void *>(ws + net->layers[idx].out_off);
}

static sol_status run_layers(sol_network *net, const void *x, void *y, void *workspace, size_t workspace_bytes,
                             int first, int last, hipStream_t st) {
    SOL_REQUIRE(net, SOL_ERR_NULL, "net is NULL");
    SOL_REQUIRE(x && y, SOL_ERR_NULL, "x and y must not be NULL");
    SOL_REQUIRE(workspace || net->ws_bytes == 0, SOL_ERR_NULL, "workspace is NULL");
    SOL_REQUIRE(workspace_bytes >= net->ws_bytes, SOL_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, net->ws_bytes);
    SOL_REQUIRE(aligned16(x) && aligned16(y) && aligned16(workspace), SOL_ERR_ALIGN, "device pointers must be 16-byte aligned");
    const int nl = (int)net->layers.size();
    SOL_REQUIRE(first >= 0 && first <= last && last < nl, SOL_ERR_SHAPE, "bad layer range [%d,%d]", first, last);
    for (int i = first; i <= last; i++) {
        const LayerPlan &lp = net->layers[i];
        if (lp.L.kind == SOL_LAYER_CONV || lp.L.kind == SOL_LAYER_LINEAR)
            SOL_REQUIRE(lp.params_set, SOL_ERR_WORKSPACE, "layer %d: parameters not set", i);
    }
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    for (int i = first; i <= last; i++) {
        const LayerPlan &lp = net->layers[i];
        const void *in = layer_in(net, lp.src, x, ws);
        void *out = i + 1 == nl ? y : static_cast<void *>(ws + lp.out_off);
        switch (lp.L.kind) {
            case SOL_LAYER_CONV: {
                const float *scale = reinterpret_cast<const float *>(net->params + lp.scale_off);
                const float *shift = reinterpret_cast<const float *>(net->params + lp.shift_off);
                const void *res = lp.res >= 0 ? layer_in(net, lp.res, x, ws) : nullptr;
                void *conv_dst = lp.split_pool ? static_cast<void *>(ws + lp.tmp_off) : out;
                SOL_TRY(conv_fused_impl(lp.in, in, lp.cd, net->params + lp.w_off, scale, shift, res, lp.L.act,
                                        lp.fuse_pool ? &lp.L.pool : nullptr, conv_dst, nullptr, nullptr, g_tile_override, st));
                if (lp.split_pool) SOL_TRY(pool_impl(lp.conv_out, conv_dst, lp.L.pool, out, nullptr, st));
                break;
            }
            case SOL_LAYER_LINEAR: {
                const float *shift = reinterpret_cast<const float *>(net->params + lp.shift_off);
                SOL_TRY(conv_fused_impl(lp.in, in, lp.cd, net->params + lp.w_off, nullptr, shift, nullptr, lp.L.act, nullptr,
                                        out, nullptr, nullptr, g_tile_override, st));
                break;
            }
            case SOL_LAYER_POOL: SOL_TRY(pool_impl(lp.in, in, lp.L.pool, out, nullptr, st)); break;
            case SOL_LAYER_GAP:
                if (lp.in.n > 0) SOL_TRY(launch_gap(in, out, lp.in.n, lp.in.h * lp.in.w, lp.in.c, lp.in.dtype, st));
                break;
        }
    }
    return SOL_OK;
}

sol_status sol_network_forward(sol_network *net, const void *x, void *y, void *workspace, size_t workspace_bytes, void *stream) {
    SOL_REQUIRE(net, SOL_ERR_NULL, "net is NULL");
    return run_layers(net, x, y, workspace, workspace_bytes, 0, (int)net->layers.size() - 1, (hipStream_t)stream);
}

sol_status sol_network_run_layer(sol_network *net, int layer, const void *x, void *y, void *workspace,
                                 size_t workspace_bytes, void *stream) {
    return run_layers(net, x, y, workspace, workspace_bytes, layer, layer, (hipStream_t)stream);
}

sol_status sol_network_layer_output(const sol_network *net, int layer, void *workspace, void **ptr) {
    SOL_REQUIRE(net && workspace && ptr, SOL_ERR_NULL, "net, workspace and ptr must not be NULL");
    SOL_REQUIRE(layer >= 0 && layer + 1 < (int)net->layers.size(), SOL_ERR_SHAPE,
                "layer %d has no workspace buffer (the last layer writes to y)", layer);
    *ptr = static_cast<unsigned char *>(workspace) + net->layers[layer].out_off;
    return SOL_OK;
}

}  // extern "C"

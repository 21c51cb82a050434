// Memory-bound kernels of the fusion engine: pooling, global average pooling, and the one-off
// parameter preparation (weight packing, BN folding).  No matrix cores here: every kernel is one
// coalesced NHWC pass with 16-byte accesses along the channel axis, the MI355X form of the paper's
// fused loop nests for all non-contraction layers (Sec. III-A, depth-first fusion module; Sec. IV,
// AveragePooling listing for the pooling semantics).
#include <math.h>

#include "common.h"
#include "vec_io.h"

namespace sol {

// ---- parameter preparation ------------------------------------------------------------------------
template <typename T>
__global__ void pack_weights_kernel(const float *__restrict__ w, T *__restrict__ out, int K, int C, int R,
                                    int S, int Kp, int Kr, int Cr) {
    // w holds Kr x Cr filters (Kr <= K, Cr <= C): output and input channels the planner added as padding are zero
    const long total = (long)K * Kp;
    for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
        const int k = (int)(i / Kp), j = (int)(i % Kp);
        float v = 0.f;
        if (j < R * S * C) {
            const int c = j % C, tap = j / C, s = tap % S, r = tap / S;
            if (k < Kr && c < Cr) v = w[(((long)k * Cr + c) * R + r) * S + s];
        }
        Elem<T>::store(out + i, v);
    }
}

template <typename T>
__global__ void unpack_weights_kernel(const T *__restrict__ in, float *__restrict__ w, int K, int C, int R,
                                      int S, int Kp) {
    const long total = (long)K * C * R * S;
    for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
        const int s = (int)(i % S);
        long t = i / S;
        const int r = (int)(t % R); t /= R;
        const int c = (int)(t % C);
        const int k = (int)(t / C);
        w[i] = Elem<T>::load(in + (long)k * Kp + ((long)r * S + s) * C + c);
    }
}

__global__ void fold_bn_kernel(int c, const float *gamma, const float *beta, const float *mean, const float *var,
                               const float *bias, float eps, float *scale, float *shift) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= c) return;
    const float b = bias ? bias[i] : 0.f;
    if (gamma) {
        const float sc = gamma[i] / sqrtf(var[i] + eps);
        scale[i] = sc;
        shift[i] = beta[i] - mean[i] * sc + b * sc;
    } else {
        scale[i] = 1.f;
        shift[i] = b;
    }
}

// ---- pooling ----------------------------------------------------------------------------------------
// One thread = one output pixel x V consecutive channels; consecutive lanes walk the channel axis
// first, so every window tap is one coalesced 16-byte-per-lane access.
template <typename T, int V>
__global__ void __launch_bounds__(256) pool_kernel(const PoolArgs a) {
    const int cg = a.C / V;
    const long total = (long)a.N * a.Ho * a.Wo * cg;
    const T *__restrict__ x = static_cast<const T *>(a.x);
    T *__restrict__ y = static_cast<T *>(a.y);
    for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
        const int g = (int)(i % cg);
        long t = i / cg;
        const int q = (int)(t % a.Wo); t /= a.Wo;
        const int p = (int)(t % a.Ho);
        const int n = (int)(t / a.Ho);
        float best[V];
        int bi[V];
#pragma unroll
        for (int e = 0; e < V; e++) { best[e] = 0.f; bi[e] = -1; }
        int cnt = 0;
        for (int r = 0; r < a.kh; r++) {
            const int ih = p * a.sh + r - a.ph;
            if ((unsigned)ih >= (unsigned)a.H) continue;
            for (int s = 0; s < a.kw; s++) {
                const int iw = q * a.sw + s - a.pw;
                if ((unsigned)iw >= (unsigned)a.W) continue;
                float v[V];
                VecIO<T, V>::load(x + (((long)n * a.H + ih) * a.W + iw) * a.C + g * V, v);
                cnt++;
                if (a.kind == SOL_POOL_MAX) {
                    // row-major window scan, strict '>' : the first of equal maxima wins
#pragma unroll
                    for (int e = 0; e < V; e++)
                        if (bi[e] < 0 || v[e] > best[e]) { best[e] = v[e]; bi[e] = ih * a.W + iw; }
                } else {
#pragma unroll
                    for (int e = 0; e < V; e++) best[e] += v[e];
                }
            }
        }
        if (a.kind == SOL_POOL_AVG) {
            const float div = a.count_pad ? (float)(a.kh * a.kw) : (float)cnt;
#pragma unroll
            for (int e = 0; e < V; e++) best[e] = best[e] / div;
        }
        const long o = i * V;   // == (((n*Ho+p)*Wo+q)*C + g*V)
        VecIO<T, V>::store(y + o, best);
        if (a.argmax && a.kind == SOL_POOL_MAX) {
#pragma unroll
            for (int e = 0; e < V; e++) a.argmax[o + e] = bi[e];
        }
    }
}

// Tiled variant for overlapping windows (kernel > stride): a workgroup owns a 4 x 8 block of output
// pixels (all channels), so the rows and columns that neighbouring windows share are re-read from
// its own L1, and consecutive workgroup ids -- which the hardware deals round-robin to the 8 XCDs --
// are remapped so that every XCD works on one contiguous run of blocks: window halos shared between
// blocks are then found in that XCD's L2 instead of being fetched from HBM once per XCD.
// ARG: the argmax is wanted (max pool only); without it the maximum is a plain v_max per element.
template <typename T, int V, bool ARG>
__global__ void __launch_bounds__(256) pool_tiled_kernel(const PoolArgs a, int tiles_h, int tiles_w, int nblocks) {
    constexpr int TH = 4, TW = 8;
    const int per_xcd = (nblocks + 7) >> 3;
    const int blk = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if (blk >= nblocks) return;
    const int tw = blk % tiles_w, t2 = blk / tiles_w;
    const int th = t2 % tiles_h, n = t2 / tiles_h;
    const int cg = a.C / V;
    const T *__restrict__ x = static_cast<const T *>(a.x);
    T *__restrict__ y = static_cast<T *>(a.y);
    for (int it = threadIdx.x; it < TH * TW * cg; it += 256) {
        const int g = it % cg, pix = it / cg;
        const int p = th * TH + pix / TW, q = tw * TW + pix % TW;
        if (p >= a.Ho || q >= a.Wo) continue;
        float best[V];
        int bi[V];
#pragma unroll
        for (int e = 0; e < V; e++) { best[e] = (!ARG && a.kind == SOL_POOL_MAX) ? -INFINITY : 0.f; bi[e] = -1; }
        int cnt = 0;
        for (int r = 0; r < a.kh; r++) {
            const int ih = p * a.sh + r - a.ph;
            if ((unsigned)ih >= (unsigned)a.H) continue;
            for (int s = 0; s < a.kw; s++) {
                const int iw = q * a.sw + s - a.pw;
                if ((unsigned)iw >= (unsigned)a.W) continue;
                float v[V];
                VecIO<T, V>::load(x + (((long)n * a.H + ih) * a.W + iw) * a.C + g * V, v);
                cnt++;
                if (a.kind == SOL_POOL_MAX && ARG) {
#pragma unroll
                    for (int e = 0; e < V; e++)
                        if (bi[e] < 0 || v[e] > best[e]) { best[e] = v[e]; bi[e] = ih * a.W + iw; }
                } else if (a.kind == SOL_POOL_MAX) {
#pragma unroll
                    for (int e = 0; e < V; e++) best[e] = fmaxf(best[e], v[e]);
                } else {
#pragma unroll
                    for (int e = 0; e < V; e++) best[e] += v[e];
                }
            }
        }
        if (a.kind == SOL_POOL_AVG) {
            const float div = a.count_pad ? (float)(a.kh * a.kw) : (float)cnt;
#pragma unroll
            for (int e = 0; e < V; e++) best[e] = best[e] / div;
        }
        const long o = ((((long)n * a.Ho + p) * a.Wo + q) * cg + g) * V;
        VecIO<T, V>::store(y + o, best);
        if (ARG && a.argmax && a.kind == SOL_POOL_MAX) {
#pragma unroll
            for (int e = 0; e < V; e++) a.argmax[o + e] = bi[e];
        }
    }
}

// Compile-time window, unconditional loads: out-of-image taps read a clamped (valid) address and are
// masked afterwards, so all KH*KW 16-byte loads of a thread are independent and in flight together --
// with one load at a time the kernel is bound by memory latency, not bandwidth.
template <typename T, int V, int KH, int KW, bool ARG>
__global__ void __launch_bounds__(256) pool_window_kernel(const PoolArgs a, int tiles_h, int tiles_w, int nblocks) {
    constexpr int TH = 4, TW = 8;
    const int per_xcd = (nblocks + 7) >> 3;
    const int blk = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if (blk >= nblocks) return;
    const int tw = blk % tiles_w, t2 = blk / tiles_w;
    const int th = t2 % tiles_h, n = t2 / tiles_h;
    const int cg = a.C / V;
    const T *__restrict__ x = static_cast<const T *>(a.x);
    T *__restrict__ y = static_cast<T *>(a.y);
    for (int it = threadIdx.x; it < TH * TW * cg; it += 256) {
        const int g = it % cg, pix = it / cg;
        const int p = th * TH + pix / TW, q = tw * TW + pix % TW;
        if (p >= a.Ho || q >= a.Wo) continue;
        const int ih0 = p * a.sh - a.ph, iw0 = q * a.sw - a.pw;
        const T *base = x + (long)n * a.H * a.W * a.C + g * V;
        uint4 raw[KH * KW];
        unsigned okmask = 0;
#pragma unroll
        for (int r = 0; r < KH; r++)
#pragma unroll
            for (int s = 0; s < KW; s++) {
                const int ih = ih0 + r, iw = iw0 + s;
                if ((unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W) okmask |= 1u << (r * KW + s);
                const int ch = min(max(ih, 0), a.H - 1), cw = min(max(iw, 0), a.W - 1);
                raw[r * KW + s] = *reinterpret_cast<const uint4 *>(base + ((long)ch * a.W + cw) * a.C);
            }
        float best[V];
        int bi[V];
#pragma unroll
        for (int e = 0; e < V; e++) { best[e] = (!ARG && a.kind == SOL_POOL_MAX) ? -INFINITY : 0.f; bi[e] = -1; }
#pragma unroll
        for (int k = 0; k < KH * KW; k++) {
            const bool ok = (okmask >> k) & 1u;
            float v[V];
            VecIO<T, V>::unpack(raw[k], v);
            if (a.kind == SOL_POOL_MAX && ARG) {
                const int idx = (ih0 + k / KW) * a.W + iw0 + k % KW;
#pragma unroll
                for (int e = 0; e < V; e++)
                    if (ok && (bi[e] < 0 || v[e] > best[e])) { best[e] = v[e]; bi[e] = idx; }
            } else if (a.kind == SOL_POOL_MAX) {
#pragma unroll
                for (int e = 0; e < V; e++) best[e] = fmaxf(best[e], ok ? v[e] : -INFINITY);
            } else {
#pragma unroll
                for (int e = 0; e < V; e++) best[e] += ok ? v[e] : 0.f;
            }
        }
        if (a.kind == SOL_POOL_AVG) {
            const float div = a.count_pad ? (float)(KH * KW) : (float)__builtin_popcount(okmask);
#pragma unroll
            for (int e = 0; e < V; e++) best[e] = best[e] / div;
        }
        const long o = ((((long)n * a.Ho + p) * a.Wo + q) * cg + g) * V;
        VecIO<T, V>::store(y + o, best);
        if (ARG && a.argmax && a.kind == SOL_POOL_MAX) {
#pragma unroll
            for (int e = 0; e < V; e++) a.argmax[o + e] = bi[e];
        }
    }
}

template <typename T, int V>
static void launch_pool_t(const PoolArgs &a, hipStream_t st) {
    const long total = (long)a.N * a.Ho * a.Wo * (a.C / V);
    if (total <= 0) return;
    long blocks = (total + 255) / 256;
    if (blocks > 256L * 64) blocks = 256L * 64;
    if (a.kh > a.sh || a.kw > a.sw) {             // overlapping windows: tiled, XCD-aware
        const int tiles_h = ceil_div(a.Ho, 4), tiles_w = ceil_div(a.Wo, 8);
        const int nb = a.N * tiles_h * tiles_w;
        if (V > 1 && a.kh == 3 && a.kw == 3) {
            if (a.argmax && a.kind == SOL_POOL_MAX)
                hipLaunchKernelGGL((pool_window_kernel<T, V, 3, 3, true>), dim3((unsigned)(((nb + 7) / 8) * 8)), dim3(256), 0, st, a, tiles_h, tiles_w, nb);
            else
                hipLaunchKernelGGL((pool_window_kernel<T, V, 3, 3, false>), dim3((unsigned)(((nb + 7) / 8) * 8)), dim3(256), 0, st, a, tiles_h, tiles_w, nb);
            return;
        }
        if (a.argmax && a.kind == SOL_POOL_MAX)
            hipLaunchKernelGGL((pool_tiled_kernel<T, V, true>), dim3((unsigned)(((nb + 7) / 8) * 8)), dim3(256), 0, st, a, tiles_h, tiles_w, nb);
        else
            hipLaunchKernelGGL((pool_tiled_kernel<T, V, false>), dim3((unsigned)(((nb + 7) / 8) * 8)), dim3(256), 0, st, a, tiles_h, tiles_w, nb);
        return;
    }
    hipLaunchKernelGGL((pool_kernel<T, V>), dim3((unsigned)blocks), dim3(256), 0, st, a);
}

sol_status launch_pool(const PoolArgs &a, int dt, hipStream_t st) {
    if (dt == SOL_BF16) {
        if (a.C % 8 == 0) launch_pool_t<bf16_t, 8>(a, st); else launch_pool_t<bf16_t, 1>(a, st);
    } else {
        if (a.C % 4 == 0) launch_pool_t<float, 4>(a, st); else launch_pool_t<float, 1>(a, st);
    }
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

// ---- global average pool ------------------------------------------------------------------------------
// One wavefront-row of lanes walks the channel axis (coalesced), SPLIT lanes-rows of a block share the
// H*W axis and combine through LDS; the sum runs in fp32.
template <typename T, int V>
__global__ void __launch_bounds__(256) gap_kernel(const T *__restrict__ x, T *__restrict__ y, int N, int HW, int C) {
    constexpr int SPLIT = 16, CGB = 16;            // 16 channel-vectors x 16 pixel slices per block: the tensor is small
    __shared__ float part[SPLIT][CGB][V + 1];      // (7-26 MB here), so the job is to have enough loads in flight chip-wide
    const int cg = C / V;
    const int gblocks = (cg + CGB - 1) / CGB;
    const int n = blockIdx.x / gblocks;
    const int lg = threadIdx.x % CGB, slice = threadIdx.x / CGB;
    const int g = (blockIdx.x % gblocks) * CGB + lg;
    float acc[V];
#pragma unroll
    for (int e = 0; e < V; e++) acc[e] = 0.f;
    if (g < cg) {
        const T *p = x + (long)n * HW * C + g * V;
        int i = slice;
        for (; i + 3 * SPLIT < HW; i += 4 * SPLIT) {          // four independent loads per trip, added in pixel order
            float v[4][V];
#pragma unroll
            for (int u = 0; u < 4; u++) VecIO<T, V>::load(p + (long)(i + u * SPLIT) * C, v[u]);
#pragma unroll
            for (int u = 0; u < 4; u++)
#pragma unroll
                for (int e = 0; e < V; e++) acc[e] += v[u][e];
        }
        for (; i < HW; i += SPLIT) {
            float v[V];
            VecIO<T, V>::load(p + (long)i * C, v);
#pragma unroll
            for (int e = 0; e < V; e++) acc[e] += v[e];
        }
    }
#pragma unroll
    for (int e = 0; e < V; e++) part[slice][lg][e] = acc[e];
    __syncthreads();
    if (slice == 0 && g < cg) {
        float o[V];
#pragma unroll
        for (int e = 0; e < V; e++) {
            float t = part[0][lg][e];
#pragma unroll
            for (int s2 = 1; s2 < SPLIT; s2++) t += part[s2][lg][e];   // fixed order
            o[e] = t / (float)HW;
        }
        VecIO<T, V>::store(y + (long)n * C + g * V, o);
    }
}

template <typename T, int V> static void launch_gap_t(const void *x, void *y, int N, int HW, int C, hipStream_t st) {
    const int gblocks = (C / V + 15) / 16;
    if (N * gblocks <= 0) return;
    hipLaunchKernelGGL((gap_kernel<T, V>), dim3(N * gblocks), dim3(256), 0, st, static_cast<const T *>(x),
                       static_cast<T *>(y), N, HW, C);
}

sol_status launch_gap(const void *x, void *y, int N, int HW, int C, int dt, hipStream_t st) {
    if (dt == SOL_BF16) {
        if (C % 8 == 0) launch_gap_t<bf16_t, 8>(x, y, N, HW, C, st); else launch_gap_t<bf16_t, 1>(x, y, N, HW, C, st);
    } else {
        if (C % 4 == 0) launch_gap_t<float, 4>(x, y, N, HW, C, st); else launch_gap_t<float, 1>(x, y, N, HW, C, st);
    }
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

// One part of a channel concatenation: x [rows][cv] -> y [rows][ldv] at column offv, in units of V.  The planner
// lets the producers write their slices themselves whenever it can; this copy is for the parts it cannot (a
// producer with other consumers, a pool or a depthwise layer in front, kept activations).
template <typename V>
__global__ void __launch_bounds__(256) concat_copy_kernel(const V *__restrict__ x, V *__restrict__ y, long total, int cv, int ldv, int offv) {
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const long r = i / cv;
        const int c = (int)(i - r * cv);
        y[r * ldv + offv + c] = x[i];
    }
}

sol_status launch_concat_copy(const void *x, void *y, long rows, int c, int ldy, int off, int dt, hipStream_t st) {
    if (rows <= 0 || c <= 0) return SOL_OK;
    const int es = (int)dtype_size(dt);
    auto go = [&](auto tag, int unit) {
        using V = decltype(tag);
        const long total = rows * (c * es / unit);
        long blocks = (total + 255) / 256;
        if (blocks > 16384) blocks = 16384;
        hipLaunchKernelGGL(concat_copy_kernel<V>, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<const V *>(x), static_cast<V *>(y),
                           total, c * es / unit, ldy * es / unit, off * es / unit);
    };
    if ((c * es) % 16 == 0 && (ldy * es) % 16 == 0 && (off * es) % 16 == 0) go(uint4{}, 16);
    else if (es == 4) go(uint32_t{}, 4);
    else go(uint16_t{}, 2);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

sol_status launch_pack(const sol_conv_desc &cd, int dt, const float *w, void *out, bool unpack, hipStream_t st, int cout_real, int cin_real) {
    const int Kr = cout_real > 0 ? cout_real : cd.cout, Cr = cin_real > 0 ? cin_real : cd.cin;
    const int Kp = packed_k(cd, dt);
    const long total = unpack ? (long)cd.cout * cd.cin * cd.kh * cd.kw : (long)cd.cout * Kp;
    if (total <= 0) return SOL_OK;
    long blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    if (dt == SOL_BF16) {
        if (unpack)
            hipLaunchKernelGGL((unpack_weights_kernel<bf16_t>), dim3((unsigned)blocks), dim3(256), 0, st,
                               static_cast<const bf16_t *>(out), const_cast<float *>(w), cd.cout, cd.cin, cd.kh, cd.kw, Kp);
        else
            hipLaunchKernelGGL((pack_weights_kernel<bf16_t>), dim3((unsigned)blocks), dim3(256), 0, st, w,
                               static_cast<bf16_t *>(out), cd.cout, cd.cin, cd.kh, cd.kw, Kp, Kr, Cr);
    } else {
        if (unpack)
            hipLaunchKernelGGL((unpack_weights_kernel<float>), dim3((unsigned)blocks), dim3(256), 0, st,
                               static_cast<const float *>(out), const_cast<float *>(w), cd.cout, cd.cin, cd.kh, cd.kw, Kp);
        else
            hipLaunchKernelGGL((pack_weights_kernel<float>), dim3((unsigned)blocks), dim3(256), 0, st, w,
                               static_cast<float *>(out), cd.cout, cd.cin, cd.kh, cd.kw, Kp, Kr, Cr);
    }
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

sol_status launch_fold(int c, const float *gamma, const float *beta, const float *mean, const float *var,
                       const float *bias, float eps, float *scale, float *shift, hipStream_t st) {
    if (c <= 0) return SOL_OK;
    hipLaunchKernelGGL(fold_bn_kernel, dim3((c + 255) / 256), dim3(256), 0, st, c, gamma, beta, mean, var, bias, eps,
                       scale, shift);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

}  // namespace sol

// Depthwise convolution in the fusion engine.  A grouped convolution with as many groups as channels has
// no reduction over channels: every output element is a weighted sum over its own channel's window, i.e. a
// pooling layer with learned per-channel window weights (Sec. III-A: such convolutions are handed to the
// depth-first module instead of the contraction libraries).  So it runs here as one coalesced NHWC pass --
// 16-byte accesses along the channel axis, fp32 accumulation, and the folded batch-norm / bias, residual
// and ReLU applied before the single store -- and never touches the matrix cores.
#include <algorithm>

#include "common.h"
#include "vec_io.h"

namespace sol {

// fp32 [C][1][kh][kw] (framework layout) -> [kh*kw][C] in T: one 16-byte load fetches a tap's weights for
// the V channels a thread owns.
template <typename T>
__global__ void pack_dw_kernel(const float *__restrict__ w, T *__restrict__ out, int C, int taps) {
    const int total = C * taps;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
        const int c = i % C, tap = i / C;
        Elem<T>::store(out + i, w[(long)c * taps + tap]);
    }
}

template <typename T, int V>
__device__ __forceinline__ void dw_epilogue(const DwArgs &a, const float acc[V], long o, int c0) {
    float v[V];
#pragma unroll
    for (int e = 0; e < V; e++) v[e] = acc[e];
    if (a.scale) {
#pragma unroll
        for (int e = 0; e < V; e++) v[e] *= a.scale[c0 + e];
    }
    if (a.shift) {
#pragma unroll
        for (int e = 0; e < V; e++) v[e] += a.shift[c0 + e];
    }
    if (a.res) {
        float r[V];
        VecIO<T, V>::load(static_cast<const T *>(a.res) + o, r);
#pragma unroll
        for (int e = 0; e < V; e++) v[e] += r[e];
    }
    if (a.act == SOL_ACT_RELU) {
#pragma unroll
        for (int e = 0; e < V; e++) v[e] = fmaxf(v[e], 0.f);
    }
    VecIO<T, V>::store(static_cast<T *>(a.y) + o, v);
}

// Any window, any stride, any channel count: one thread = one output pixel x V channels.
template <typename T, int V>
__global__ void __launch_bounds__(256) dwconv_kernel(const DwArgs a) {
    const int cg = a.C / V;
    const long total = (long)a.N * a.Ho * a.Wo * cg;
    const T *__restrict__ x = static_cast<const T *>(a.x);
    const T *__restrict__ w = static_cast<const T *>(a.w);
    for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
        const int g = (int)(i % cg);
        long t = i / cg;
        const int q = (int)(t % a.Wo); t /= a.Wo;
        const int p = (int)(t % a.Ho);
        const int n = (int)(t / a.Ho);
        float acc[V];
#pragma unroll
        for (int e = 0; e < V; e++) acc[e] = 0.f;
        for (int r = 0; r < a.kh; r++) {
            const int ih = p * a.sh + r - a.ph;
            if ((unsigned)ih >= (unsigned)a.H) continue;
            for (int s = 0; s < a.kw; s++) {
                const int iw = q * a.sw + s - a.pw;
                if ((unsigned)iw >= (unsigned)a.W) continue;
                float xv[V], wv[V];
                VecIO<T, V>::load(x + (((long)n * a.H + ih) * a.W + iw) * a.C + g * V, xv);
                VecIO<T, V>::load(w + (long)(r * a.kw + s) * a.C + g * V, wv);
#pragma unroll
                for (int e = 0; e < V; e++) acc[e] = fmaf(xv[e], wv[e], acc[e]);
            }
        }
        dw_epilogue<T, V>(a, acc, i * V, g * V);
    }
}

// Compile-time window and horizontal stride.  A thread owns V channels of a strip of TQ consecutive output
// pixels of one row: neighbouring windows share columns, so the strip needs (TQ-1)*SW+KW input columns per
// filter row instead of TQ*KW, and the filter's KH*KW weight vectors are fetched once per strip.  Loads are
// unconditional -- taps outside the image read a clamped address and are zeroed afterwards -- so a whole
// filter row of 16-byte loads is in flight at once.  A workgroup takes TH rows x TS strips x all channels
// (sizes chosen per layer by the launcher); consecutive workgroup ids, which the hardware deals round-robin
// to the 8 XCDs, are remapped so that each XCD works on one contiguous run of tiles and the rows shared by
// vertically adjacent tiles are found in that XCD's L2.
template <typename T, int V, int KH, int KW, int SW, int TQ>
__global__ void __launch_bounds__(256) dwconv_strip_kernel(const DwArgs a, int TH, int TS, int tiles_h, int tiles_w,
                                                           int nblocks, FastDiv dcg, FastDiv dts) {
    constexpr int NCOL = (TQ - 1) * SW + KW;
    const int per_xcd = (nblocks + 7) >> 3;
    const int blk = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if (blk >= nblocks) return;
    const int tw = blk % tiles_w, t2 = blk / tiles_w;
    const int th = t2 % tiles_h, n = t2 / tiles_h;
    const int cg = a.C / V;
    const T *__restrict__ x = static_cast<const T *>(a.x) + (long)n * a.H * a.W * a.C;
    const T *__restrict__ w = static_cast<const T *>(a.w);
    const int items = TH * TS * cg;
    for (int it = threadIdx.x; it < items; it += 256) {
        uint32_t rest, g, prow, strip;
        dcg.divmod((uint32_t)it, rest, g);
        dts.divmod(rest, prow, strip);
        const int p = th * TH + (int)prow, q0 = (tw * TS + (int)strip) * TQ;
        if (p >= a.Ho || q0 >= a.Wo) continue;
        const int ih0 = p * a.sh - a.ph, iw0 = q0 * SW - a.pw;
        const T *xb = x + g * V;
        uint4 wraw[KH * KW];
#pragma unroll
        for (int k = 0; k < KH * KW; k++) wraw[k] = *reinterpret_cast<const uint4 *>(w + (long)k * a.C + g * V);
        float acc[TQ][V];
#pragma unroll
        for (int t = 0; t < TQ; t++)
#pragma unroll
            for (int e = 0; e < V; e++) acc[t][e] = 0.f;
        int cw[NCOL];
        unsigned colok = 0;
#pragma unroll
        for (int c = 0; c < NCOL; c++) {
            const int iw = iw0 + c;
            if ((unsigned)iw < (unsigned)a.W) colok |= 1u << c;
            cw[c] = min(max(iw, 0), a.W - 1) * a.C;
        }
#pragma unroll
        for (int r = 0; r < KH; r++) {
            const int ih = ih0 + r;
            const bool rowok = (unsigned)ih < (unsigned)a.H;
            const T *xr = xb + (long)min(max(ih, 0), a.H - 1) * a.W * a.C;
            uint4 raw[NCOL];
#pragma unroll
            for (int c = 0; c < NCOL; c++) raw[c] = *reinterpret_cast<const uint4 *>(xr + cw[c]);
            float xv[NCOL][V];
#pragma unroll
            for (int c = 0; c < NCOL; c++) {
                const bool ok = rowok && ((colok >> c) & 1u);
                const uint4 z = ok ? raw[c] : make_uint4(0u, 0u, 0u, 0u);
                VecIO<T, V>::unpack(z, xv[c]);
            }
#pragma unroll
            for (int s = 0; s < KW; s++) {
                float wv[V];
                VecIO<T, V>::unpack(wraw[r * KW + s], wv);
#pragma unroll
                for (int t = 0; t < TQ; t++)
#pragma unroll
                    for (int e = 0; e < V; e++) acc[t][e] = fmaf(xv[t * SW + s][e], wv[e], acc[t][e]);
            }
        }
        const long o0 = ((((long)n * a.Ho + p) * a.Wo + q0) * cg + g) * V;
#pragma unroll
        for (int t = 0; t < TQ; t++)
            if (q0 + t < a.Wo) dw_epilogue<T, V>(a, acc[t], o0 + (long)t * a.C, (int)g * V);
    }
}

template <typename T, int V, int KH, int KW, int SW, int TQ>
static void launch_strip(const DwArgs &a, hipStream_t st) {
    const int cg = a.C / V, strips = ceil_div(a.Wo, TQ);
    // about two work items per thread and workgroup; whole rows of strips first, then rows
    int TS = std::min(strips, std::max(1, 512 / cg));
    if (TS * 2 > strips && TS < strips) TS = ceil_div(strips, 2);          // avoid a thin last tile column
    int TH = std::min(std::min(a.Ho, 8), std::max(1, ceil_div(512, TS * cg)));
    const int tiles_h = ceil_div(a.Ho, TH), tiles_w = ceil_div(strips, TS);
    const int nb = a.N * tiles_h * tiles_w;
    hipLaunchKernelGGL((dwconv_strip_kernel<T, V, KH, KW, SW, TQ>), dim3((unsigned)(((nb + 7) / 8) * 8)), dim3(256), 0, st, a,
                       TH, TS, tiles_h, tiles_w, nb, FastDiv((uint32_t)cg), FastDiv((uint32_t)TS));
}

template <typename T, int V>
static void launch_dw_t(const DwArgs &a, hipStream_t st) {
    if constexpr (V > 1) {
        if (a.kh == 3 && a.kw == 3 && a.sw == 1) return launch_strip<T, V, 3, 3, 1, 4>(a, st);
        if (a.kh == 3 && a.kw == 3 && a.sw == 2) return launch_strip<T, V, 3, 3, 2, 2>(a, st);
    }
    const long total = (long)a.N * a.Ho * a.Wo * (a.C / V);
    long blocks = (total + 255) / 256;
    if (blocks > 256L * 64) blocks = 256L * 64;
    hipLaunchKernelGGL((dwconv_kernel<T, V>), dim3((unsigned)blocks), dim3(256), 0, st, a);
}

sol_status launch_dwconv(const DwArgs &a, int dt, hipStream_t st) {
    if ((long)a.N * a.Ho * a.Wo * a.C <= 0) return SOL_OK;
    if (dt == SOL_BF16) {
        if (a.C % 8 == 0) launch_dw_t<bf16_t, 8>(a, st); else launch_dw_t<bf16_t, 1>(a, st);
    } else {
        if (a.C % 4 == 0) launch_dw_t<float, 4>(a, st); else launch_dw_t<float, 1>(a, st);
    }
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

sol_status launch_pack_dw(int C, int taps, int dt, const float *w, void *out, hipStream_t st) {
    const long total = (long)C * taps;
    if (total <= 0) return SOL_OK;
    const unsigned blocks = (unsigned)std::min<long>((total + 255) / 256, 4096);
    if (dt == SOL_BF16)
        hipLaunchKernelGGL((pack_dw_kernel<bf16_t>), dim3(blocks), dim3(256), 0, st, w, static_cast<bf16_t *>(out), C, taps);
    else
        hipLaunchKernelGGL((pack_dw_kernel<float>), dim3(blocks), dim3(256), 0, st, w, static_cast<float *>(out), C, taps);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

}  // namespace sol

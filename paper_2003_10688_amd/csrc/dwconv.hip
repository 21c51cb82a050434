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

// 3x3 window, strides 1 and 2.  The arithmetic, not HBM, is what limits a depthwise convolution on this chip:
// 9 multiply-adds per output element against 4 bytes moved (bf16), with every bf16 operand costing one more
// VALU operation to widen.  So the kernel is built to widen each input element once and each weight once per
// thread: a thread owns 4 channels of a strip of TQ output columns and walks DOWN the image, keeping the three
// input rows its current output row needs as fp32 registers (3 x NCOL x 4 values).  Moving to the next output
// row loads only the SH new input rows -- issued before the current row's arithmetic so the loads are covered by
// it -- and the 36 filter values and the per-channel scale / shift stay in registers for the whole walk.  The
// row loop is unrolled by 3 so that the window's row slots rotate by renaming, not by copies.  Loads are
// unconditional (clamped address, zeroed afterwards when outside the image).  4 channels per thread (8-byte
// accesses for bf16) rather than 8 keeps the window within the register file at TQ = 4.
template <typename T> struct Quad;          // 4 consecutive channels of one pixel
template <> struct Quad<float> {
    typedef uint4 raw_t;
    static __device__ __forceinline__ raw_t zero() { return make_uint4(0u, 0u, 0u, 0u); }
    static __device__ __forceinline__ void unpack(const raw_t &u, float v[4]) {
        v[0] = __uint_as_float(u.x); v[1] = __uint_as_float(u.y); v[2] = __uint_as_float(u.z); v[3] = __uint_as_float(u.w);
    }
    static __device__ __forceinline__ void store(float *p, const float v[4]) { *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]); }
};
template <> struct Quad<bf16_t> {
    typedef uint2 raw_t;
    static __device__ __forceinline__ raw_t zero() { return make_uint2(0u, 0u); }
    static __device__ __forceinline__ void unpack(const raw_t &u, float v[4]) {
        v[0] = __uint_as_float(u.x << 16); v[1] = __uint_as_float(u.x & 0xffff0000u);
        v[2] = __uint_as_float(u.y << 16); v[3] = __uint_as_float(u.y & 0xffff0000u);
    }
    static __device__ __forceinline__ void store(bf16_t *p, const float v[4]) {
        *reinterpret_cast<uint2 *>(p) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
    }
};

template <typename T, int SH, int SW, int TQ>
__global__ void __launch_bounds__(256) dwconv_walk_kernel(const DwArgs a, int RT, uint32_t nitems, FastDiv dcg, FastDiv dstrips,
                                                          FastDiv dchunks) {
    typedef typename Quad<T>::raw_t raw_t;
    constexpr int V = 4, NCOL = (TQ - 1) * SW + 3;
    const uint32_t nblocks = (nitems + 255u) >> 8, per_xcd = (nblocks + 7u) >> 3;
    const uint32_t blk = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
    const uint32_t item = blk * 256u + threadIdx.x;
    if (blk >= nblocks || item >= nitems) return;
    uint32_t rest, g, strip, n, chunk;
    dcg.divmod(item, rest, g);
    dstrips.divmod(rest, rest, strip);
    dchunks.divmod(rest, n, chunk);
    const int p0 = (int)chunk * RT, nrows = min(RT, a.Ho - p0), q0 = (int)strip * TQ;
    const int c0 = (int)g * V;
    const T *__restrict__ xb = static_cast<const T *>(a.x) + (long)n * a.H * a.W * a.C + c0;
    const T *__restrict__ w = static_cast<const T *>(a.w) + c0;

    float wv[9][V], sc[V], sf[V];
#pragma unroll
    for (int k = 0; k < 9; k++) Quad<T>::unpack(*reinterpret_cast<const raw_t *>(w + (long)k * a.C), wv[k]);
#pragma unroll
    for (int e = 0; e < V; e++) { sc[e] = a.scale ? a.scale[c0 + e] : 1.f; sf[e] = a.shift ? a.shift[c0 + e] : 0.f; }

    int coff[NCOL];
    unsigned colok = 0;
#pragma unroll
    for (int c = 0; c < NCOL; c++) {
        const int iw = q0 * SW - a.pw + c;
        if ((unsigned)iw < (unsigned)a.W) colok |= 1u << c;
        coff[c] = min(max(iw, 0), a.W - 1) * a.C;
    }
    const int ih_base = p0 * SH - a.ph;        // input row of window row 0 of the chunk's first output row
    const int rowpitch = a.W * a.C;
    float win[3][NCOL][V];
    // input row j of the chunk (image row ih_base + j) -> raw registers / -> window slot
    auto fetch = [&](int j, raw_t raw[NCOL]) {
        const T *xr = xb + (long)min(max(ih_base + j, 0), a.H - 1) * rowpitch;
#pragma unroll
        for (int c = 0; c < NCOL; c++) raw[c] = *reinterpret_cast<const raw_t *>(xr + coff[c]);
    };
    auto widen = [&](int j, const raw_t raw[NCOL], float dst[NCOL][V]) {
        const bool rowok = (unsigned)(ih_base + j) < (unsigned)a.H;
#pragma unroll
        for (int c = 0; c < NCOL; c++) {
            const raw_t z = (rowok && ((colok >> c) & 1u)) ? raw[c] : Quad<T>::zero();
            Quad<T>::unpack(z, dst[c]);
        }
    };
    {
        raw_t raw[3][NCOL];
#pragma unroll
        for (int j = 0; j < 3; j++) fetch(j, raw[j]);
#pragma unroll
        for (int j = 0; j < 3; j++) widen(j, raw[j], win[j]);
    }
    T *__restrict__ y = static_cast<T *>(a.y);
    const T *__restrict__ res = static_cast<const T *>(a.res);
    for (int k0 = 0; k0 < nrows; k0 += 3) {
#pragma unroll
        for (int u = 0; u < 3; u++) {
            const int k = k0 + u;
            if (k < nrows) {
                // the SH input rows that output row k+1 adds to the window
                raw_t raw[SH][NCOL];
#pragma unroll
                for (int i = 0; i < SH; i++) fetch((k + 1) * SH + 3 - SH + i, raw[i]);
                float acc[TQ][V];
#pragma unroll
                for (int t = 0; t < TQ; t++)
#pragma unroll
                    for (int e = 0; e < V; e++) acc[t][e] = 0.f;
#pragma unroll
                for (int r = 0; r < 3; r++)
#pragma unroll
                    for (int s2 = 0; s2 < 3; s2++)
#pragma unroll
                        for (int t = 0; t < TQ; t++)
#pragma unroll
                            for (int e = 0; e < V; e++)
                                acc[t][e] = fmaf(win[(u * SH + r) % 3][t * SW + s2][e], wv[r * 3 + s2][e], acc[t][e]);
                const long o0 = (((long)n * a.Ho + p0 + k) * a.Wo + q0) * a.C + c0;
#pragma unroll
                for (int t = 0; t < TQ; t++) {
                    if (q0 + t < a.Wo) {
                        float v[V];
#pragma unroll
                        for (int e = 0; e < V; e++) v[e] = fmaf(acc[t][e], sc[e], sf[e]);
                        if (res) {
                            float rv[V];
                            Quad<T>::unpack(*reinterpret_cast<const raw_t *>(res + o0 + (long)t * a.C), rv);
#pragma unroll
                            for (int e = 0; e < V; e++) v[e] += rv[e];
                        }
                        if (a.act == SOL_ACT_RELU) {
#pragma unroll
                            for (int e = 0; e < V; e++) v[e] = fmaxf(v[e], 0.f);
                        }
                        Quad<T>::store(y + o0 + (long)t * a.C, v);
                    }
                }
#pragma unroll
                for (int i = 0; i < SH; i++) widen((k + 1) * SH + 3 - SH + i, raw[i], win[(u * SH + i) % 3]);
            }
        }
    }
}

template <typename T, int SH, int SW, int TQ>
static void launch_walk(const DwArgs &a, hipStream_t st) {
    const int cg = a.C / 4, strips = ceil_div(a.Wo, TQ);
    // rows per thread: long walks amortise the two halo rows (16 measured best on the large layers), small layers
    // are cut further until the chip has a wave per SIMD; the rows are then dealt evenly over the chunks
    const long columns = (long)a.N * cg * strips;
    const int want_chunks = (int)std::min<long>(std::max(1, a.Ho / 2), std::max<long>(1, (1024L * 64 + columns - 1) / columns));
    const int chunks0 = std::max(ceil_div(a.Ho, 16), want_chunks);
    const int RT = ceil_div(a.Ho, chunks0), chunks = ceil_div(a.Ho, RT);
    const uint32_t nitems = (uint32_t)(columns * chunks);
    const uint32_t nb = (nitems + 255u) / 256u;
    hipLaunchKernelGGL((dwconv_walk_kernel<T, SH, SW, TQ>), dim3(((nb + 7u) / 8u) * 8u), dim3(256), 0, st, a, RT, nitems,
                       FastDiv((uint32_t)cg), FastDiv((uint32_t)strips), FastDiv((uint32_t)chunks));
}

template <typename T, int V>
static void launch_dw_t(const DwArgs &a, hipStream_t st) {
    if (a.kh == 3 && a.kw == 3 && a.C % 4 == 0 && a.sh == a.sw && (a.sh == 1 || a.sh == 2)) {
        if (a.sh == 1) return launch_walk<T, 1, 1, 4>(a, st);
        return launch_walk<T, 2, 2, 2>(a, st);
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

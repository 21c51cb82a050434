// Fused implicit-GEMM convolution for gfx950 (MI355X).
//
// Computes the fused block of the library's problem statement,
//     y = pool( act( scale[k] * conv(x, w)[., k] + shift[k] + residual ) ),
// as one dense contraction on the matrix cores with the memory-bound neighbours applied to the
// accumulators in registers, so that no pre-BN / pre-ReLU intermediate ever reaches HBM (the
// "keep data in registers and caches" principle of the paper's fusion module, Sec. III-A, applied
// to the contraction layers the paper hands to a vendor library).
//
// GEMM view:  D[k][m] = sum_j  Wp[k][j] * Xg[m][j]
//   m  = output pixel (n, p, q)           -> MFMA column (one pixel per lane)
//   k  = output channel                   -> MFMA row (4 consecutive channels per lane register group)
//   j  = (r, s, c) reduction index        -> contiguous in NHWC activations and in the packed weights
// so a lane owns 4 consecutive channels of one pixel and stores them with one vector store.
//
// Both operands are staged through LDS in rows of 128 bytes (64 bf16 / 32 fp32 reduction elements)
// whose eight 16-byte chunks are XOR-swizzled with the row index, which makes both the 16-byte
// tile stores and the 16-byte MFMA fragment reads bank-conflict free.  Global loads for the next
// reduction chunk are issued before the MFMAs of the current one (register prefetch) and two LDS
// buffers alternate, so there is one barrier per chunk.
#include "common.h"

namespace sol {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

template <typename T> struct Mma;
template <> struct Mma<bf16_t> {
    // one v_mfma_f32_32x32x16_bf16: each lane supplies 8 consecutive reduction elements
    static __device__ __forceinline__ void run(f32x16_t &acc, const uint4 &a, const uint4 &b) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                      __builtin_bit_cast(bf16x8_t, b), acc, 0, 0, 0);
    }
};
template <> struct Mma<float> {
    // four v_mfma_f32_32x32x2_f32 (true fp32 multiplies); the reduction order inside a 128-byte row
    // is permuted identically for both operands, which leaves the sum unchanged
    static __device__ __forceinline__ void run(f32x16_t &acc, const uint4 &a, const uint4 &b) {
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
    }
};

// GEMM row m -> output pixel.  With a fused 2x2 pool the rows are ordered window-major, so that the
// four elements of one pooling window sit in four adjacent lanes in row-major window order.
__device__ __forceinline__ void decode_pixel(const ConvArgs &a, int m, int &n, int &op, int &oq) {
    if (a.pool) {
        const int win = m >> 2, d = m & 3;
        const int qp = win % a.Wy, t = win / a.Wy;
        const int pp = t % a.Hy;
        n = t / a.Hy;
        op = 2 * pp + (d >> 1);
        oq = 2 * qp + (d & 1);
    } else {
        oq = m % a.Wo;
        const int t = m / a.Wo;
        op = t % a.Ho;
        n = t / a.Ho;
    }
}

template <typename T> __device__ __forceinline__ void store_vec4(T *p, const float v[4]);
template <> __device__ __forceinline__ void store_vec4<float>(float *p, const float v[4]) {
    *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
template <> __device__ __forceinline__ void store_vec4<bf16_t>(bf16_t *p, const float v[4]) {
    uint2 u;
    u.x = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
    u.y = (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16);
    *reinterpret_cast<uint2 *>(p) = u;
}
template <typename T> __device__ __forceinline__ void load_vec4(const T *p, float v[4]);
template <> __device__ __forceinline__ void load_vec4<float>(const float *p, float v[4]) {
    const float4 f = *reinterpret_cast<const float4 *>(p);
    v[0] = f.x; v[1] = f.y; v[2] = f.z; v[3] = f.w;
}
template <> __device__ __forceinline__ void load_vec4<bf16_t>(const bf16_t *p, float v[4]) {
    const uint2 u = *reinterpret_cast<const uint2 *>(p);
    v[0] = __uint_as_float(u.x << 16); v[1] = __uint_as_float(u.x & 0xffff0000u);
    v[2] = __uint_as_float(u.y << 16); v[3] = __uint_as_float(u.y & 0xffff0000u);
}

// nv = number of valid channels among the 4 (0..4); vec = Cout % 4 == 0
template <typename T>
__device__ __forceinline__ void store4(T *p, const float v[4], int nv, bool vec) {
    if (nv <= 0) return;
    if (vec) { store_vec4<T>(p, v); return; }
    for (int e = 0; e < 4; e++)
        if (e < nv) Elem<T>::store(p + e, v[e]);
}
template <typename T>
__device__ __forceinline__ void load4(const T *p, float v[4], int nv, bool vec) {
    if (nv <= 0) { v[0] = v[1] = v[2] = v[3] = 0.f; return; }
    if (vec) { load_vec4<T>(p, v); return; }
    for (int e = 0; e < 4; e++) v[e] = e < nv ? Elem<T>::load(p + e) : 0.f;
}

// T: element type; BP x BC: pixels x channels per workgroup; WP x WC: wave grid;
// VEC: every 128-byte reduction chunk lies inside one filter tap (Cin % BK == 0) and is fetched with
// 16-byte loads; otherwise (small Cin, e.g. 3) elements are gathered one by one.
template <typename T, int BP, int BC, int WP, int WC, bool VEC>
__global__ void __launch_bounds__(WP *WC * 64) conv_igemm_kernel(const ConvArgs a) {
    constexpr int NT = WP * WC * 64;
    constexpr int BK = 128 / (int)sizeof(T);   // reduction elements per LDS row
    constexpr int EPC = 16 / (int)sizeof(T);   // elements per 16-byte chunk
    constexpr int TP = BP / (WP * 32), TC = BC / (WC * 32);
    constexpr int RPP = NT / 8;                // tile rows covered by one pass of 16-byte loads
    constexpr int XA = VEC ? BP / RPP : 1, XB = BC / RPP;
    constexpr int RG = NT / BK;                // rows per pass of the element-wise gather
    constexpr int XG = VEC ? 1 : BP / RG;
    static_assert(BP % RPP == 0 && BC % RPP == 0 && BP % (WP * 32) == 0 && BC % (WC * 32) == 0, "tile");
    static_assert(NT % BK == 0 && BP % RG == 0, "gather tile");

    __shared__ __align__(16) unsigned char lds[2 * (BP + BC) * 128];
    __shared__ int row_base[BP], row_ih0[BP], row_iw0[BP];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wp = wave % WP, wc = wave / WP;

    // XCD-aware tile order: consecutive workgroup ids go round-robin over the 8 XCDs, so give each
    // XCD one contiguous run of tiles (neighbouring pixel tiles and all channel tiles of a pixel
    // tile then share that XCD's L2).
    const int per_xcd = (a.ntiles + 7) >> 3;
    const int tile = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if (tile >= a.ntiles) return;
    const int p0 = (tile / a.ntc) * BP, c0 = (tile % a.ntc) * BC;

    const T *__restrict__ xg = static_cast<const T *>(a.x);
    const T *__restrict__ wg = static_cast<const T *>(a.w);

    for (int r = tid; r < BP; r += NT) {
        const int m = p0 + r;
        int base = 0, ih0 = -(1 << 20), iw0 = -(1 << 20);
        if (m < a.P) {
            int n, op, oq;
            decode_pixel(a, m, n, op, oq);
            ih0 = op * a.sh - a.ph;
            iw0 = oq * a.sw - a.pw;
            base = ((n * a.H + ih0) * a.W + iw0) * a.C;
        }
        row_base[r] = base; row_ih0[r] = ih0; row_iw0[r] = iw0;
    }
    __syncthreads();

    // ---- loader state ---------------------------------------------------------------------------
    const int lchunk = tid & 7, lrow = tid >> 3;
    int rb[XA], rh[XA], rw[XA];
    if (VEC) {
#pragma unroll
        for (int i = 0; i < XA; i++) {
            const int r = lrow + i * RPP;
            rb[i] = row_base[r] + lchunk * EPC; rh[i] = row_ih0[r]; rw[i] = row_iw0[r];
        }
    }
    int wb[XB];
#pragma unroll
    for (int i = 0; i < XB; i++) {
        const int co = c0 + lrow + i * RPP;
        wb[i] = co < a.Cout ? co * a.Kp + lchunk * EPC : -1;
    }
    const int gk = tid % BK, grow = tid / BK;   // gather mapping (non-VEC)

    uint4 ra[XA], rwt[XB];
    T rg[XG];
    const int cpt = VEC ? a.C / BK : 1;         // chunks per filter tap
    const int nk = VEC ? a.R * a.S * cpt : a.Kp / BK;
    int tr = 0, ts = 0, tcc = 0;                // tap row / tap column / chunk inside tap of the NEXT load

    auto load_tiles = [&](int kc) {
        if (VEC) {
            const int tapoff = (tr * a.W + ts) * a.C + tcc * BK;
#pragma unroll
            for (int i = 0; i < XA; i++) {
                const bool ok = (unsigned)(rh[i] + tr) < (unsigned)a.H && (unsigned)(rw[i] + ts) < (unsigned)a.W;
                ra[i] = ok ? *reinterpret_cast<const uint4 *>(xg + (rb[i] + tapoff)) : make_uint4(0, 0, 0, 0);
            }
            if (++tcc == cpt) { tcc = 0; if (++ts == a.S) { ts = 0; ++tr; } }
        } else {
            const int k = kc * BK + gk;
            const int c = k % a.C, tap = k / a.C;
            const int s = tap % a.S, r = tap / a.S;
            const bool kok = k < a.Ktot;
            const int tapoff = (r * a.W + s) * a.C + c;
#pragma unroll
            for (int i = 0; i < XG; i++) {
                const int row = grow + i * RG;
                const bool ok = kok && (unsigned)(row_ih0[row] + r) < (unsigned)a.H &&
                                (unsigned)(row_iw0[row] + s) < (unsigned)a.W;
                rg[i] = ok ? xg[row_base[row] + tapoff] : (T)0;
            }
        }
#pragma unroll
        for (int i = 0; i < XB; i++)
            rwt[i] = wb[i] >= 0 ? *reinterpret_cast<const uint4 *>(wg + (wb[i] + kc * BK)) : make_uint4(0, 0, 0, 0);
    };

    auto store_tiles = [&](int buf) {
        unsigned char *lx = lds + buf * (BP + BC) * 128, *lw = lx + BP * 128;
        if (VEC) {
#pragma unroll
            for (int i = 0; i < XA; i++) {
                const int row = lrow + i * RPP;
                *reinterpret_cast<uint4 *>(lx + row * 128 + ((lchunk ^ (row & 7)) << 4)) = ra[i];
            }
        } else {
            const int gchunk = gk / EPC, gin = (gk % EPC) * (int)sizeof(T);
#pragma unroll
            for (int i = 0; i < XG; i++) {
                const int row = grow + i * RG;
                *reinterpret_cast<T *>(lx + row * 128 + ((gchunk ^ (row & 7)) << 4) + gin) = rg[i];
            }
        }
#pragma unroll
        for (int i = 0; i < XB; i++) {
            const int row = lrow + i * RPP;
            *reinterpret_cast<uint4 *>(lw + row * 128 + ((lchunk ^ (row & 7)) << 4)) = rwt[i];
        }
    };

    f32x16_t acc[TC][TP];
#pragma unroll
    for (int i = 0; i < TC; i++)
#pragma unroll
        for (int j = 0; j < TP; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

    const int lr = lane & 31, lh = lane >> 5;

    load_tiles(0);
    store_tiles(0);
    __syncthreads();
    for (int kc = 0; kc < nk; kc++) {
        const int buf = kc & 1;
        if (kc + 1 < nk) load_tiles(kc + 1);
        const unsigned char *lx = lds + buf * (BP + BC) * 128, *lw = lx + BP * 128;
#pragma unroll
        for (int ks = 0; ks < 4; ks++) {
            const int sw = ((2 * ks + lh) ^ (lr & 7)) << 4;
            uint4 fa[TC], fb[TP];
#pragma unroll
            for (int i = 0; i < TC; i++)
                fa[i] = *reinterpret_cast<const uint4 *>(lw + (wc * TC * 32 + i * 32 + lr) * 128 + sw);
#pragma unroll
            for (int j = 0; j < TP; j++)
                fb[j] = *reinterpret_cast<const uint4 *>(lx + (wp * TP * 32 + j * 32 + lr) * 128 + sw);
#pragma unroll
            for (int i = 0; i < TC; i++)
#pragma unroll
                for (int j = 0; j < TP; j++) Mma<T>::run(acc[i][j], fa[i], fb[j]);
        }
        if (kc + 1 < nk) store_tiles(buf ^ 1);
        __syncthreads();
    }

    // ---- fused epilogue: affine (folded BN + bias), residual, activation, optional 2x2 pool -------
    T *__restrict__ yg = static_cast<T *>(a.y);
    const T *__restrict__ resg = static_cast<const T *>(a.res);
    T *__restrict__ preg = static_cast<T *>(a.prepool);
    const bool vec = (a.Cout & 3) == 0;
#pragma unroll
    for (int j = 0; j < TP; j++) {
        const int m = p0 + wp * TP * 32 + j * 32 + lr;
        const bool mok = m < a.P;
        long opix = m;          // pixel index in the conv-output NHWC tensor
        int pp = 0, qp = 0;
        if (a.pool) {
            int n = 0, op = 0, oq = 0;
            if (mok) decode_pixel(a, m, n, op, oq);
            opix = ((long)n * a.Ho + op) * a.Wo + oq;
            pp = op >> 1; qp = oq >> 1;
        }
#pragma unroll
        for (int i = 0; i < TC; i++) {
#pragma unroll
            for (int g = 0; g < 4; g++) {
                const int co = c0 + wc * TC * 32 + i * 32 + 8 * g + 4 * lh;
                const int nv = mok ? min(4, a.Cout - co) : 0;
                float v[4], sc[4] = {1.f, 1.f, 1.f, 1.f}, sf[4] = {0.f, 0.f, 0.f, 0.f};
                if (a.scale) load4<float>(a.scale + co, sc, nv, vec);
                if (a.shift) load4<float>(a.shift + co, sf, nv, vec);
#pragma unroll
                for (int e = 0; e < 4; e++) v[e] = acc[i][j][4 * g + e] * sc[e] + sf[e];
                if (resg) {
                    float rv[4];
                    load4<T>(resg + opix * a.Cout + co, rv, nv, vec);
#pragma unroll
                    for (int e = 0; e < 4; e++) v[e] += rv[e];
                }
                if (a.act == SOL_ACT_RELU) {
#pragma unroll
                    for (int e = 0; e < 4; e++) v[e] = v[e] > 0.f ? v[e] : 0.f;
                }
                if (!a.pool) {
                    store4<T>(yg + (long)m * a.Cout + co, v, nv, vec);
                } else {
                    if (preg) store4<T>(preg + opix * a.Cout + co, v, nv, vec);
                    // the 4 window elements live in the 4 lanes of a quad, in row-major window order
                    const int q0 = lane & ~3;
                    float o[4];
                    int oi[4];
#pragma unroll
                    for (int e = 0; e < 4; e++) {
                        const float w0 = __shfl(v[e], q0), w1 = __shfl(v[e], q0 + 1);
                        const float w2 = __shfl(v[e], q0 + 2), w3 = __shfl(v[e], q0 + 3);
                        if (a.pool == 1) {
                            float best = w0; int bi = 0;
                            if (w1 > best) { best = w1; bi = 1; }
                            if (w2 > best) { best = w2; bi = 2; }
                            if (w3 > best) { best = w3; bi = 3; }
                            o[e] = best; oi[e] = bi;
                        } else {
                            o[e] = (((w0 + w1) + w2) + w3) * 0.25f; oi[e] = 0;
                        }
                    }
                    if ((lane & 3) == 0 && nv > 0) {
                        const long obase = (long)(m >> 2) * a.Cout + co;
                        store4<T>(yg + obase, o, nv, vec);
                        if (a.argmax && a.pool == 1) {
                            for (int e = 0; e < 4; e++)
                                if (e < nv)
                                    a.argmax[obase + e] = (2 * pp + (oi[e] >> 1)) * a.Wo + 2 * qp + (oi[e] & 1);
                        }
                    }
                }
            }
        }
    }
}

// ---- launcher / tile table ------------------------------------------------------------------------
template <typename T, int BP, int BC, int WP, int WC, bool VEC>
static sol_status launch_cfg(ConvArgs a, hipStream_t st) {
    a.ntc = ceil_div(a.Cout, BC);
    a.ntiles = ceil_div(a.P, BP) * a.ntc;
    const int grid = ((a.ntiles + 7) / 8) * 8;
    hipLaunchKernelGGL((conv_igemm_kernel<T, BP, BC, WP, WC, VEC>), dim3(grid), dim3(WP * WC * 64), 0, st, a);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

// tile ids (also accepted as a debugging override): pixels x channels per workgroup
enum { T_AUTO = 0, T_256x128 = 1, T_128x128 = 2, T_128x64 = 3, T_256x64 = 4, T_64x64 = 5, T_128x32 = 6,
       T_128x256 = 7, T_64x128 = 8, T_COUNT };

static int choose_tile(const ConvArgs &a, bool vec) {
    if (!vec) return a.Cout <= 32 ? T_128x32 : T_128x64;
    if (a.Cout <= 32) return T_128x32;
    const long cus = 256;
    if (a.Cout <= 64) return ((long)ceil_div(a.P, 256) >= 2 * cus) ? T_256x64 : (ceil_div(a.P, 128) >= cus ? T_128x64 : T_64x64);
    auto tiles = [&](int bp, int bc) { return (long)ceil_div(a.P, bp) * ceil_div(a.Cout, bc); };
    if (tiles(256, 128) >= 2 * cus) return T_256x128;
    if (tiles(128, 128) >= 2 * cus) return T_128x128;
    if (tiles(64, 128) >= cus) return T_64x128;
    return T_64x64;
}

template <typename T> static sol_status launch_typed(const ConvArgs &a, int tile, hipStream_t st) {
    constexpr int BK = 128 / (int)sizeof(T);
    const bool vec = a.C % BK == 0;
    if (tile == T_AUTO) tile = choose_tile(a, vec);
    if (!vec) {
        switch (tile) {
            case T_128x32: return launch_cfg<T, 128, 32, 4, 1, false>(a, st);
            default: return launch_cfg<T, 128, 64, 2, 2, false>(a, st);
        }
    }
    switch (tile) {
        case T_256x128: return launch_cfg<T, 256, 128, 2, 2, true>(a, st);
        case T_128x128: return launch_cfg<T, 128, 128, 2, 2, true>(a, st);
        case T_128x64: return launch_cfg<T, 128, 64, 2, 2, true>(a, st);
        case T_256x64: return launch_cfg<T, 256, 64, 4, 1, true>(a, st);
        case T_64x64: return launch_cfg<T, 64, 64, 2, 2, true>(a, st);
        case T_128x32: return launch_cfg<T, 128, 32, 4, 1, true>(a, st);
        case T_128x256: return launch_cfg<T, 128, 256, 2, 2, true>(a, st);
        case T_64x128: return launch_cfg<T, 64, 128, 2, 2, true>(a, st);
        default: SOL_FAIL(SOL_ERR_UNSUPPORTED, "unknown conv tile id %d", tile);
    }
}

sol_status launch_conv(const ConvArgs &a, int dt, int tile_override, hipStream_t st) {
    if (a.P <= 0) return SOL_OK;   // empty batch: nothing to do
    if (dt == SOL_BF16) return launch_typed<bf16_t>(a, tile_override, st);
    if (dt == SOL_F32) return launch_typed<float>(a, tile_override, st);
    SOL_FAIL(SOL_ERR_DTYPE, "unknown dtype %d", dt);
}

}  // namespace sol

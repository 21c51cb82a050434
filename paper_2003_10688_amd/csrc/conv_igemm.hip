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
// so the accumulators of a lane are 4 consecutive channels of one pixel; the epilogue transposes
// them through LDS into rows of 8 channels per lane and writes whole 128-byte lines.
//
// Both operands are staged through LDS in rows of 128 bytes (64 bf16 / 32 fp32 reduction elements)
// whose eight 16-byte chunks are XOR-swizzled with the row index, which makes both the 16-byte
// tile stores and the 16-byte MFMA fragment reads bank-conflict free.  Global loads for the next
// reduction chunk are issued before the MFMAs of the current one (register prefetch) and two LDS
// buffers alternate, so there is one barrier per chunk.
#include "conv_common.h"

namespace sol {

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
    static_assert(XA <= 32 && XG <= 32, "one validity bit per staged row");

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
            base = ((n * a.H + ih0) * a.W + iw0) * a.ldx;
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
    // input-side BN + ReLU: the per-channel constants of the chunk being fetched, and which of its rows are real data
    const bool pre = a.pre_scale != nullptr;
    const bool partial = a.Cvalid < a.C;                  // channels >= Cvalid are whatever memory holds: they must read as 0
    float psc[EPC], psh[EPC];
    unsigned okm = 0, cfirst = 0;                        // VEC: bit i = row i of ra[] is in range; first channel of this lane's 16 bytes
    float gsc = 0.f, gsh = 0.f;                          // gather path: constants of this lane's reduction element
    bool gvalid = true;
    const int cpt = VEC ? a.C / BK : 1;         // chunks per filter tap
    const int nk = VEC ? a.R * a.S * cpt : a.Kp / BK;
    int tr = 0, ts = 0, tcc = 0;                // tap row / tap column / chunk inside tap of the NEXT load

    auto load_tiles = [&](int kc) {
        if (VEC) {
            const int tapoff = (tr * a.W + ts) * a.ldx + tcc * BK;
            okm = 0;
#pragma unroll
            for (int i = 0; i < XA; i++) {
                const bool ok = (unsigned)(rh[i] + tr) < (unsigned)a.H && (unsigned)(rw[i] + ts) < (unsigned)a.W;
                ra[i] = ok ? *reinterpret_cast<const uint4 *>(xg + (rb[i] + tapoff)) : make_uint4(0, 0, 0, 0);
                okm |= ok ? 1u << i : 0u;
            }
            cfirst = (unsigned)(tcc * BK + lchunk * EPC);
            if (pre) {
#pragma unroll
                for (int e = 0; e < EPC; e += 4) {
                    const float4 s4 = *reinterpret_cast<const float4 *>(a.pre_scale + cfirst + e), h4 = *reinterpret_cast<const float4 *>(a.pre_shift + cfirst + e);
                    psc[e] = s4.x; psc[e + 1] = s4.y; psc[e + 2] = s4.z; psc[e + 3] = s4.w;
                    psh[e] = h4.x; psh[e + 1] = h4.y; psh[e + 2] = h4.z; psh[e + 3] = h4.w;
                }
            }
            if (++tcc == cpt) { tcc = 0; if (++ts == a.S) { ts = 0; ++tr; } }
        } else {
            const int k = kc * BK + gk;
            const int c = k % a.C, tap = k / a.C;
            const int s = tap % a.S, r = tap / a.S;
            const bool kok = k < a.Ktot;
            const int tapoff = (r * a.W + s) * a.ldx + c;
            gvalid = c < a.Cvalid;
            okm = 0;
            if (pre) { gsc = kok ? a.pre_scale[c] : 0.f; gsh = kok ? a.pre_shift[c] : 0.f; }
#pragma unroll
            for (int i = 0; i < XG; i++) {
                const int row = grow + i * RG;
                const bool ok = kok && (unsigned)(row_ih0[row] + r) < (unsigned)a.H &&
                                (unsigned)(row_iw0[row] + s) < (unsigned)a.W;
                rg[i] = ok ? xg[row_base[row] + tapoff] : (T)0;
                okm |= ok ? 1u << i : 0u;
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
                uint4 v = ra[i];
                if (pre || partial) {                     // wave-uniform
                    T *el = reinterpret_cast<T *>(&v);
                    const bool ok = (okm >> i) & 1u;
#pragma unroll
                    for (int e = 0; e < EPC; e++) {
                        float f = Elem<T>::load(el + e);
                        if (pre) { f = f * psc[e] + psh[e]; f = __builtin_fmaxf(f, 0.f); }
                        f = (ok && (int)(cfirst + e) < a.Cvalid) ? f : 0.f;       // padding taps and padding channels are zeros, not relu(shift)
                        Elem<T>::store(el + e, f);
                    }
                }
                *reinterpret_cast<uint4 *>(lx + row * 128 + ((lchunk ^ ((row >> 1) & 7)) << 4)) = v;
            }
        } else {
            const int gchunk = gk / EPC, gin = (gk % EPC) * (int)sizeof(T);
#pragma unroll
            for (int i = 0; i < XG; i++) {
                const int row = grow + i * RG;
                T v = rg[i];
                if (pre || partial) {
                    float f = Elem<T>::load(&v);
                    if (pre) { f = f * gsc + gsh; f = __builtin_fmaxf(f, 0.f); }
                    f = (((okm >> i) & 1u) && gvalid) ? f : 0.f;
                    Elem<T>::store(&v, f);
                }
                *reinterpret_cast<T *>(lx + row * 128 + ((gchunk ^ ((row >> 1) & 7)) << 4) + gin) = v;
            }
        }
#pragma unroll
        for (int i = 0; i < XB; i++) {
            const int row = lrow + i * RPP;
            *reinterpret_cast<uint4 *>(lw + row * 128 + ((lchunk ^ ((row >> 1) & 7)) << 4)) = rwt[i];
        }
    };

    const Affine8 aff = load_affine<TC>(a, lane, c0 + wc * TC * 32);
    ResidualRegs<T, TP, TC> resregs;
    prefetch_residual<T, TP, TC>(a, lane, p0 + wp * TP * 32, c0 + wc * TC * 32, LinearRows{a.P}, resregs);
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
            const int sw = ((2 * ks + lh) ^ ((lr >> 1) & 7)) << 4;
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

    static_assert((WP * WC) * 32 * (TC * 32 + 4) * 4 <= 2 * (BP + BC) * 128, "epilogue strip must fit in the tile buffers");
    conv_epilogue_auto<T, TP, TC>(a, acc, reinterpret_cast<float *>(lds), wave, lane, p0 + wp * TP * 32, c0 + wc * TC * 32, aff, LinearRows{a.P}, resregs);
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

// Planner heuristic: tile per layer shape, from per-layer timing sweeps on MI355X.  Small-Cin layers
// use the element-gather kernel; everything else the LDS-DMA ring kernel with
//   - 64x64 tiles (many resident workgroups) for narrow outputs and for layers with few tiles,
//   - 128x64 / 64x64 tiles, 64-byte rows x 4 stages (3-5 workgroups per CU) for the big HBM-bound layers,
//   - 128x128 tiles, 128-byte rows x 2 stages for the mid-sized, reuse-heavy layers.
// The LDS-DMA kernel keeps one validity bit per filter tap in a 32-bit mask and addresses both
// operands with 32-bit byte offsets.
static bool dma_kernel_applies(const ConvArgs &a, int esize) {
    const double xb = (double)a.N * a.H * a.W * a.C * esize + (double)(a.ph * a.W + a.pw) * a.C * esize;
    return a.R * a.S <= 32 && xb < 4294967296.0 && (double)a.Cout * a.Kp * esize < 4294967296.0;
}

static int choose_tile(const ConvArgs &a, int esize) {
    const bool dma_ok = dma_kernel_applies(a, esize);
    const bool dma128 = dma_ok && a.C % (128 / esize) == 0, dma64 = dma_ok && a.C % (64 / esize) == 0;
    if (a.Cout <= 32 || !dma64) return a.C % (128 / esize) == 0 ? (a.Cout <= 32 ? T_128x32 : T_128x64)
                                                                 : (a.Cout <= 32 ? T_128x32 : T_128x64);
    const bool wide = a.R * a.S > 1;
    if (a.Cout <= 64) return (wide && dma128) ? D_64x64_128x3 : D_64x64_64x4;
    const long nt = (long)ceil_div(a.P, 128) * ceil_div(a.Cout, 128);
    if (nt >= 1024) return a.res ? D_64x64_64x4 : D_128x64_64x4;   // HBM-bound: many small workgroups in flight
    if (nt >= 192) return dma128 ? D_128x128_128x2 : D_128x128_64x4;
    return dma128 ? D_64x64_128x3 : D_64x64_64x4;
}

template <typename T> static sol_status launch_typed(const ConvArgs &a, int tile, hipStream_t st) {
    constexpr int BK = 128 / (int)sizeof(T);
    const bool vec = a.C % BK == 0;
    if (tile == T_AUTO) tile = choose_tile(a, (int)sizeof(T));
    if (dma_tile_row_bytes(tile)) return launch_conv_dma(a, sizeof(T) == 2 ? SOL_BF16 : SOL_F32, tile, st);
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

// Input-side BN + ReLU, a strided input (channel prefix of a wider tensor) or masked padding channels: the
// register-staged kernel is the one that can transform what it fetches on its way to LDS.
static sol_status launch_conv_staged(const ConvArgs &a, int dt, int tile, hipStream_t st) {
    if (!(tile >= T_256x128 && tile <= T_64x128)) {
        SOL_REQUIRE(tile == T_AUTO || tile == T_NO_HALO, SOL_ERR_UNSUPPORTED,
                    "conv tile %d cannot apply an input-side BN + ReLU or read a channel prefix; the register-staged tiles 1..8 can", tile);
        const long np128 = ceil_div(a.P, 128);
        tile = a.Cout <= 32 ? T_128x32 : a.Cout <= 64 ? T_128x64 : (a.Cout % 256 == 0 && np128 * (a.Cout / 256) >= 512) ? T_128x256 : T_128x128;
    }
    if (dt == SOL_BF16) return launch_typed<bf16_t>(a, tile, st);
    if (dt == SOL_F32) return launch_typed<float>(a, tile, st);
    SOL_FAIL(SOL_ERR_DTYPE, "unknown dtype %d", dt);
}

sol_status launch_conv(const ConvArgs &a, int dt, int tile_override, hipStream_t st) {
    if (a.P <= 0) return SOL_OK;   // empty batch: nothing to do
    if (a.pre_scale || a.ldx != a.C || a.Cvalid != a.C) return launch_conv_staged(a, dt, tile_override, st);
    if (tile_override == T_AUTO && stem_kernel_applies(a, dt)) return launch_conv_stem(a, st);
    if (tile_override == T_AUTO && linear_kernel_applies(a, dt)) {
        // few rows, but a weight matrix of many megabytes (the MLP workload): the job is streaming the weights, which the
        // eight-wave ring kernel does with whole 128-byte lines and eight stages in flight
        const double wbytes = (double)a.Cout * a.Kp * dtype_size(dt);
        if (wbytes >= 16.0 * 1048576 && gemm8_kernel_applies(a, dt) && a.C % 64 == 0) {
            // enough workgroups for every CU: 32-row weight tiles when 64-row tiles would leave CUs idle
            if (a.C % 128 == 0 && ceil_div(a.P, 64) * ceil_div(a.Cout, 64) < 200) return launch_conv_gemm8(a, G_64x32_k4_r256, st);
            return launch_conv_gemm8(a, G_64x64_k4_deep, st);
        }
        return launch_linear(a, dt, st);
    }
    if (tile_override == T_AUTO && halo_kernel_applies(a, dt)) {
        if (const int ht = halo_choose_tile(a)) return launch_conv_halo(a, ht, st);
    }
    if (tile_override >= H_FIRST && tile_override <= H_LAST) {
        SOL_REQUIRE(halo_kernel_applies(a, dt), SOL_ERR_UNSUPPORTED,
                    "conv tile %d needs a bf16 3x3 stride-1 pad-1 convolution with Cin %% 64 == 0 and no fused pool", tile_override);
        return launch_conv_halo(a, tile_override, st);
    }
    if (tile_override >= G_FIRST && tile_override <= G_LAST) {
        SOL_REQUIRE(gemm8_kernel_applies(a, dt), SOL_ERR_UNSUPPORTED,
                    "conv tile %d needs a bf16 convolution with at most 32 filter taps and Cin %% 32 == 0", tile_override);
        return launch_conv_gemm8(a, tile_override, st);
    }
    if (tile_override == T_NO_HALO) tile_override = T_AUTO;
    if (const int rowb = dma_tile_row_bytes(tile_override)) {
        SOL_REQUIRE(a.C % (rowb / (int)dtype_size(dt)) == 0 && dma_kernel_applies(a, (int)dtype_size(dt)), SOL_ERR_UNSUPPORTED,
                    "conv tile %d needs Cin %% %d == 0, at most 32 filter taps and tensors below 4 GB", tile_override,
                    rowb / (int)dtype_size(dt));
        return launch_conv_dma(a, dt, tile_override, st);
    }
    if (dt == SOL_BF16) return launch_typed<bf16_t>(a, tile_override, st);
    if (dt == SOL_F32) return launch_typed<float>(a, tile_override, st);
    SOL_FAIL(SOL_ERR_DTYPE, "unknown dtype %d", dt);
}

}  // namespace sol

// Fused implicit-GEMM convolution, LDS-DMA pipeline (gfx950).
//
// Same GEMM view and epilogue as conv_igemm.hip, but the operand tiles travel HBM/L2 -> LDS
// directly (global_load_lds_dwordx4: every lane fetches 16 bytes, a wave instruction fills one
// contiguous 1 KB LDS segment in lane order), without passing through registers.  That frees the
// staging registers and the LDS-store issue slots, so a ring of NS stages can be kept in flight per
// workgroup and several workgroups fit on a CU: the latency of HBM is covered by bytes in flight
// instead of by occupancy alone.  This is what both regimes of a CNN layer chain need on MI355X:
// the HBM-bound 1x1 layers need ~64 KB in flight per CU, the MFMA-bound 3x3 layers need the matrix
// pipe never to wait for a tile.
//
// LDS layout of one stage: BP pixel rows then BC weight rows, ROWB bytes each (one reduction chunk).
// A row's 16-byte slots are XOR-permuted with the row index (which slot a lane's data lands in is
// fixed by the DMA, so the permutation is applied to the global address each lane reads), making the
// 16-byte MFMA fragment reads bank-conflict free.  Padding taps and rows beyond the tensor read a
// 64-byte block of zeros instead.
#include "conv_common.h"

namespace sol {

__device__ __attribute__((used)) uint4 g_zero_block[4];   // zero-initialised; never written

template <int N> __device__ __forceinline__ void wait_vmcnt() {
    // s_waitcnt with only the vector-memory counter constrained (gfx9 encoding: vmcnt = [15:14][3:0])
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// The compiler cannot tell which ring stage a fragment read touches and would make every LDS read
// wait for ALL outstanding DMA (vmcnt(0)), serialising load and compute.  The fragment reads are
// therefore issued as opaque instructions and ordered by hand: ds_read -> s_waitcnt lgkmcnt -> use.
// All of these statements are volatile, so the compiler keeps their relative order; tying a fragment
// to an empty volatile statement after the wait makes every later use depend on the wait.
typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;

template <int OFF> __device__ __forceinline__ void lds_read16_async(u32x4_t &dst, unsigned addr) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(dst) : "v"(addr), "n"(OFF));
}
template <int N> __device__ __forceinline__ void wait_lgkmcnt() {
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N));
}
__device__ __forceinline__ void landed(u32x4_t &v) { asm volatile("" : "+v"(v)); }

__device__ __forceinline__ unsigned lds_addr(const void *p) {
    return (unsigned)(size_t)(__attribute__((address_space(3))) const void *)p;
}

__device__ __forceinline__ void dma16(const void *g, unsigned char *l) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)g,
                                     (__attribute__((address_space(3))) void *)l, 16, 0, 0);
}

// T: element type; BP x BC: pixels x channels per workgroup; WP x WC: wave grid;
// ROWB: bytes of reduction data per tile row and stage (64 or 128); NS: ring stages.
// Requires Cin % (ROWB / sizeof(T)) == 0, so that every chunk lies inside one filter tap.
template <typename T, int BP, int BC, int WP, int WC, int ROWB, int NS>
__global__ void __launch_bounds__(WP *WC * 64) conv_dma_kernel(const ConvArgs a) {
    constexpr int NW = WP * WC;
    constexpr int BK = ROWB / (int)sizeof(T);      // reduction elements per stage
    constexpr int EPC = 16 / (int)sizeof(T);       // elements per 16-byte slot
    constexpr int SLOTS = ROWB / 16;               // slots per row
    constexpr int RSEG = 64 / SLOTS;               // tile rows per 1 KB DMA segment
    constexpr int XL = BP / RSEG / NW, WL = BC / RSEG / NW;   // DMA instructions per wave and stage
    constexpr int L = XL + WL;
    constexpr int STAGE = (BP + BC) * ROWB;
    constexpr int KS = ROWB / 32;                  // MFMA k-steps per stage (2 slots each)
    constexpr int TP = BP / (WP * 32), TC = BC / (WC * 32);
    static_assert(ROWB == 64 || ROWB == 128, "row bytes");
    static_assert(BP % (RSEG * NW) == 0 && BC % (RSEG * NW) == 0, "tile rows must split evenly over the waves");
    static_assert(NS >= 2 && (NS - 2) * L <= 63, "ring depth");
    static_assert(NW * 32 * (TC * 32 + 4) * 4 <= NS * STAGE, "epilogue strip must fit in the ring");

    __shared__ __align__(1024) unsigned char lds[NS * STAGE];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wp = wave % WP, wc = wave / WP;

    const int per_xcd = (a.ntiles + 7) >> 3;       // XCD-aware tile order (see conv_igemm.hip)
    const int tile = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if (tile >= a.ntiles) return;
    const int p0 = (tile / a.ntc) * BP, c0 = (tile % a.ntc) * BC;

    const T *__restrict__ xg = static_cast<const T *>(a.x);
    const T *__restrict__ wg = static_cast<const T *>(a.w);
    const T *zero = reinterpret_cast<const T *>(g_zero_block);

    // ---- this lane's share of every stage: XL pixel rows and WL weight rows, one 16-byte slot each
    const int lslot = lane % SLOTS, lrow = lane / SLOTS;
    auto swz = [](int row) { return ROWB == 128 ? ((row >> 1) & 7) : ((row >> 2) & 3); };
    int rb[XL], rh[XL], rw[XL];
#pragma unroll
    for (int i = 0; i < XL; i++) {
        const int row = (wave * XL + i) * RSEG + lrow;
        const int m = p0 + row;
        rb[i] = 0; rh[i] = -(1 << 20); rw[i] = -(1 << 20);
        if (m < a.P) {
            int n, op, oq;
            decode_pixel(a, m, n, op, oq);
            rh[i] = op * a.sh - a.ph;
            rw[i] = oq * a.sw - a.pw;
            rb[i] = ((n * a.H + rh[i]) * a.W + rw[i]) * a.C + (lslot ^ swz(row)) * EPC;
        }
    }
    int wb[WL];
#pragma unroll
    for (int i = 0; i < WL; i++) {
        const int row = (wave * WL + i) * RSEG + lrow;
        const int co = c0 + row;
        wb[i] = co < a.Cout ? co * a.Kp + (lslot ^ swz(row)) * EPC : -1;
    }

    const int cpt = a.C / BK;                      // chunks per filter tap
    const int nk = a.R * a.S * cpt;
    int tr = 0, ts = 0, tcc = 0;                   // filter tap / chunk of the NEXT stage to issue

    auto issue = [&](int kc, int buf) {
        unsigned char *lx = lds + buf * STAGE, *lw = lx + BP * ROWB;
        const int tapoff = (tr * a.W + ts) * a.C + tcc * BK;
#pragma unroll
        for (int i = 0; i < XL; i++) {
            const bool ok = (unsigned)(rh[i] + tr) < (unsigned)a.H && (unsigned)(rw[i] + ts) < (unsigned)a.W;
            dma16(ok ? xg + (rb[i] + tapoff) : zero, lx + (wave * XL + i) * 1024);
        }
#pragma unroll
        for (int i = 0; i < WL; i++)
            dma16(wb[i] >= 0 ? wg + (wb[i] + kc * BK) : zero, lw + (wave * WL + i) * 1024);
        if (++tcc == cpt) { tcc = 0; if (++ts == a.S) { ts = 0; ++tr; } }
    };

    const Affine8 aff = load_affine<TC>(a, lane, c0 + wc * TC * 32);
    f32x16_t acc[TC][TP];
#pragma unroll
    for (int i = 0; i < TC; i++)
#pragma unroll
        for (int j = 0; j < TP; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

    const int lr = lane & 31, lh = lane >> 5;
    const int fsw = swz(lr);                       // tile row bases are multiples of 32: swizzle depends on lr only
    // LDS byte offsets of this lane's fragment rows inside a stage, one per k-step
    unsigned fx[KS], fw[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
        const unsigned so = ((2 * ks + lh) ^ fsw) << 4;
        fx[ks] = lds_addr(lds) + (wp * TP * 32 + lr) * ROWB + so;
        fw[ks] = lds_addr(lds) + BP * ROWB + (wc * TC * 32 + lr) * ROWB + so;
    }

#pragma unroll
    for (int s = 0; s < NS - 1; s++)
        if (s < nk) issue(s, s);

    // fragments of one k-step; two sets alternate so that the reads of step s+1 fly under the MFMAs of step s
    u32x4_t fa[2][TC], fb[2][TP];
    auto read_frags = [&](auto SET, int ks_dyn_unused, unsigned ax, unsigned aw) {
        constexpr int set = decltype(SET)::value;
        static_for<TC>([&](auto I) { lds_read16_async<decltype(I)::value * 32 * ROWB>(fa[set][decltype(I)::value], aw); });
        static_for<TP>([&](auto J) { lds_read16_async<decltype(J)::value * 32 * ROWB>(fb[set][decltype(J)::value], ax); });
    };

    for (int kc = 0; kc < nk; kc++) {
        // stage kc has landed once at most the (NS-2) stages issued after it are outstanding
        if (kc + NS - 2 < nk) wait_vmcnt<(NS - 2) * L>(); else wait_vmcnt<0>();
        __syncthreads();                           // ... for every wave; and stage kc-1 is no longer read
        if (kc + NS - 1 < nk) issue(kc + NS - 1, (kc + NS - 1) % NS);
        const unsigned sb = (kc % NS) * STAGE;
        read_frags(std::integral_constant<int, 0>{}, 0, fx[0] + sb, fw[0] + sb);
        static_for<KS>([&](auto KSI) {
            constexpr int ks = decltype(KSI)::value, cur = ks & 1;
            if constexpr (ks + 1 < KS) {
                read_frags(std::integral_constant<int, cur ^ 1>{}, 0, fx[ks + 1] + sb, fw[ks + 1] + sb);
                wait_lgkmcnt<TC + TP>();           // LDS returns in order: all but the newest TC+TP reads are done
            } else {
                wait_lgkmcnt<0>();
            }
            static_for<TC>([&](auto I) { landed(fa[cur][decltype(I)::value]); });
            static_for<TP>([&](auto J) { landed(fb[cur][decltype(J)::value]); });
#pragma unroll
            for (int i = 0; i < TC; i++)
#pragma unroll
                for (int j = 0; j < TP; j++) Mma<T>::run(acc[i][j], fa[cur][i], fb[cur][j]);
        });
    }
    __syncthreads();                               // every wave is done with the tiles: reuse LDS as strip
    conv_epilogue<T, TP, TC>(a, acc, reinterpret_cast<float *>(lds), wave, lane, p0 + wp * TP * 32, c0 + wc * TC * 32, aff, LinearRows{a.P});
}

template <typename T, int BP, int BC, int WP, int WC, int ROWB, int NS>
static sol_status launch_dma_cfg(ConvArgs a, hipStream_t st) {
    a.ntc = ceil_div(a.Cout, BC);
    a.ntiles = ceil_div(a.P, BP) * a.ntc;
    const int grid = ((a.ntiles + 7) / 8) * 8;
    hipLaunchKernelGGL((conv_dma_kernel<T, BP, BC, WP, WC, ROWB, NS>), dim3(grid), dim3(WP * WC * 64), 0, st, a);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

template <typename T> static sol_status launch_dma_typed(const ConvArgs &a, int tile, hipStream_t st) {
    switch (tile) {
        case D_128x128_64x4: return launch_dma_cfg<T, 128, 128, 2, 2, 64, 4>(a, st);
        case D_128x128_64x3: return launch_dma_cfg<T, 128, 128, 2, 2, 64, 3>(a, st);
        case D_256x128_64x3: return launch_dma_cfg<T, 256, 128, 2, 2, 64, 3>(a, st);
        case D_128x64_64x4: return launch_dma_cfg<T, 128, 64, 2, 2, 64, 4>(a, st);
        case D_64x64_64x4: return launch_dma_cfg<T, 64, 64, 2, 2, 64, 4>(a, st);
        case D_128x256_64x3: return launch_dma_cfg<T, 128, 256, 2, 2, 64, 3>(a, st);
        case D_256x64_64x3: return launch_dma_cfg<T, 256, 64, 4, 1, 64, 3>(a, st);
        case D_64x128_64x4: return launch_dma_cfg<T, 64, 128, 2, 2, 64, 4>(a, st);
        case D_128x128_128x2: return launch_dma_cfg<T, 128, 128, 2, 2, 128, 2>(a, st);
        case D_128x128_128x3: return launch_dma_cfg<T, 128, 128, 2, 2, 128, 3>(a, st);
        case D_128x64_128x3: return launch_dma_cfg<T, 128, 64, 2, 2, 128, 3>(a, st);
        case D_64x64_128x3: return launch_dma_cfg<T, 64, 64, 2, 2, 128, 3>(a, st);
        default: SOL_FAIL(SOL_ERR_UNSUPPORTED, "unknown conv tile id %d", tile);
    }
}

// Row bytes the tile id needs (the reduction chunk must divide Cin); 0 = not a DMA tile id.
int dma_tile_row_bytes(int tile) {
    if (tile >= D_128x128_64x4 && tile <= D_64x128_64x4) return 64;
    if (tile >= D_128x128_128x2 && tile <= D_64x64_128x3) return 128;
    return 0;
}

sol_status launch_conv_dma(const ConvArgs &a, int dt, int tile, hipStream_t st) {
    if (dt == SOL_BF16) return launch_dma_typed<bf16_t>(a, tile, st);
    if (dt == SOL_F32) return launch_dma_typed<float>(a, tile, st);
    SOL_FAIL(SOL_ERR_DTYPE, "unknown dtype %d", dt);
}

}  // namespace sol

// Fused implicit-GEMM convolution, LDS-DMA pipeline (gfx950).
//
// Same GEMM view and epilogue as conv_igemm.hip, but the operand tiles travel HBM/L2 -> LDS
// directly (buffer_load_dwordx4 ... lds: every lane fetches 16 bytes, a wave instruction fills one
// contiguous 1 KB LDS segment in lane order), without passing through registers.  That frees the
// staging registers and the LDS-store issue slots, so a ring of NS stages is kept in flight per
// workgroup and several workgroups fit on a CU.
//
// LDS layout of one stage: BP pixel rows then BC weight rows, ROWB bytes each (one reduction chunk).
// A row's 16-byte slots are XOR-permuted with the row index (which slot a lane's data lands in is
// fixed by the DMA, so the permutation is applied to the address each lane fetches), making the
// 16-byte MFMA fragment reads bank-conflict free (16 lanes x 16 bytes per LDS read cycle).  Padding
// taps and rows beyond the tensor are fetched with an out-of-range buffer offset, which the hardware
// turns into zeros.
#include "conv_common.h"

namespace sol {

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

// T: element type; BP x BC: pixels x channels per workgroup; WP x WC: wave grid;
// ROWB: bytes of reduction data per tile row and stage (64 or 128); NS: ring stages.
// Requires Cin % (ROWB / sizeof(T)) == 0 (every chunk lies inside one filter tap), at most 32 filter
// taps, and tensors smaller than 4 GB (32-bit buffer offsets).
//
// Address generation is the scarce resource of the main loop: every instruction a wave spends on
// it delays the MFMAs behind it.  The DMA therefore uses buffer addressing: a per-lane byte offset
// that is computed ONCE per tile row (voffset), a wave-uniform per-stage offset for the filter tap
// and channel chunk (soffset, scalar), and the hardware range check for everything that must read
// as zero -- rows beyond the tensor carry an out-of-range offset for good, padding taps get one by
// OR-ing in a per-row bit mask of invalid taps.  One DMA costs 2 vector + 2 scalar instructions, and
// the DMA of stage kc+NS-1 is spread between the MFMAs of stage kc.
template <typename T, int BP, int BC, int WP, int WC, int ROWB, int NS>
__global__ void __launch_bounds__(WP *WC * 64) conv_dma_kernel(const ConvArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub (buffer types are device-only)
    constexpr int NW = WP * WC;
    constexpr int ES = (int)sizeof(T);
    constexpr int BK = ROWB / ES;                  // reduction elements per stage
    constexpr int SLOTS = ROWB / 16;               // 16-byte slots per row
    constexpr int RSEG = 64 / SLOTS;               // tile rows per 1 KB DMA segment
    constexpr int XL = BP / RSEG / NW, WL = BC / RSEG / NW;   // DMA instructions per wave and stage
    constexpr int L = XL + WL;
    constexpr int STAGE = (BP + BC) * ROWB;
    constexpr int KS = ROWB / 32;                  // MFMA k-steps per stage (2 slots each)
    constexpr int TP = BP / (WP * 32), TC = BC / (WC * 32);
    static_assert(ROWB == 64 || ROWB == 128, "row bytes");
    static_assert(BP % (RSEG * NW) == 0 && BC % (RSEG * NW) == 0, "tile rows must split evenly over the waves");
    static_assert(NS >= 2 && (NS - 2) * L <= 63, "ring depth is bounded by the 6-bit vmcnt");
    static_assert(NW * 32 * (TC * 32 + 4) * 4 <= NS * STAGE, "epilogue strips must fit in the ring");

    __shared__ __align__(1024) unsigned char lds[NS * STAGE];
    __shared__ __align__(256) unsigned char l2sink[NW * 256];   // write-only landing pad of the L2 warm-up loads

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wp = wave % WP, wc = wave / WP;

    // XCD-aware tile order (workgroup ids go round-robin over the 8 XCDs, each with its own L2).  Usually an XCD
    // takes a contiguous run of tiles: few pixel tiles, all their channel tiles, i.e. 1/8 of the input and all
    // of the weights.  When the weights are the larger operand the split is by channel tile instead (cpx each):
    // an XCD then reads 1/8 of the weights and all of the input, which is what fits its L2.
    const int xcd = (int)(blockIdx.x & 7);
    int tile;
    if (a.cpx > 0) {
        const int j = (int)(blockIdx.x >> 3);
        tile = (j / a.cpx) * a.ntc + xcd * a.cpx + j % a.cpx;
    } else {
        tile = xcd * ((a.ntiles + 7) >> 3) + (int)(blockIdx.x >> 3);
    }
    if (tile >= a.ntiles) return;
    const int p0 = (tile / a.ntc) * BP, c0 = (tile % a.ntc) * BC;

    // Buffer resources.  The activation resource starts `bias` bytes before the tensor so that the
    // offset of a row's window origin (which lies in the padding for border pixels) is never negative;
    // only in-range taps are ever fetched through it.
    const unsigned bias = (unsigned)((a.ph * a.W + a.pw) * a.C) * ES;
    const unsigned xbytes = (unsigned)a.N * a.H * a.W * a.C * ES, wbytes = (unsigned)a.Cout * a.Kp * ES;
    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<unsigned char *>(static_cast<const unsigned char *>(a.x)) - bias, 0, (int)(xbytes + bias), 0x00020000);
    const __amdgpu_buffer_rsrc_t wr = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.w), 0, (int)wbytes, 0x00020000);

    // Warm this XCD's L2 with the layer's weights.  Inside a network the weights of a layer are cold when
    // it starts, every workgroup streams the same rows in lock step, and each stage would stall on an
    // HBM round trip; instead the workgroups of an XCD (blockIdx & 7) first touch one dword per
    // 128-byte line of the whole packed weight array between them, all misses in flight at once.
    {
        const unsigned nx = gridDim.x >> 3;
        // with the channel split only this XCD's rows of the packed weights
        const unsigned slice = (unsigned)(a.cpx * BC * a.Kp) * ES, first = a.cpx > 0 ? min(wbytes, (unsigned)xcd * slice) : 0u;
        const unsigned lines = (a.cpx > 0 ? min(slice, wbytes - first) : wbytes) >> 7;
        const unsigned char *wbase = static_cast<const unsigned char *>(a.w) + first;
        // the touched dwords are dropped into a per-wave LDS sink (a load into a register would have to
        // be waited for, a DMA does not)
        for (unsigned l = (blockIdx.x >> 3) * (NW * 64) + tid; l < lines; l += nx * (NW * 64))
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(wbase + ((size_t)l << 7)),
                                             (__attribute__((address_space(3))) void *)(l2sink + wave * 256), 4, 0, 0);
    }

    // ---- this lane's share of every stage: XL pixel rows and WL weight rows, one 16-byte slot each
    const int lslot = lane % SLOTS, lrow = lane / SLOTS;
    auto swz = [](int row) { return ROWB == 128 ? ((row >> 1) & 7) : ((row >> 2) & 3); };
    unsigned xo[XL], xinv[XL], wo[WL];             // byte offsets; bit t of xinv = filter tap t reads padding
#pragma unroll
    for (int i = 0; i < XL; i++) {
        const int row = (wave * XL + i) * RSEG + lrow;
        const int m = p0 + row;
        xo[i] = 0xffffffffu; xinv[i] = 0;
        if (m < a.P) {
            int n, op, oq;
            decode_pixel(a, m, n, op, oq);
            const int ih0 = op * a.sh - a.ph, iw0 = oq * a.sw - a.pw;
            xo[i] = (unsigned)(((n * a.H + ih0) * a.W + iw0) * a.C) * ES + bias + (lslot ^ swz(row)) * 16;
            // taps s in [slo, shi) of every filter row r in [rlo, rhi) are inside the image
            const int slo = max(0, -iw0), shi = min(a.S, a.W - iw0), rlo = max(0, -ih0), rhi = min(a.R, a.H - ih0);
            const unsigned cval = shi > slo ? (unsigned)((1ull << shi) - 1ull) & ~((1u << slo) - 1u) : 0u;
            unsigned val = 0;
            for (int r = 0; r < a.R; r++) val |= (r >= rlo && r < rhi) ? cval << (r * a.S) : 0u;
            xinv[i] = ~val;
        }
    }
#pragma unroll
    for (int i = 0; i < WL; i++) {
        const int row = (wave * WL + i) * RSEG + lrow;
        const int co = c0 + row;
        wo[i] = co < a.Cout ? (unsigned)(co * a.Kp) * ES + (lslot ^ swz(row)) * 16 : 0xffffffffu;
    }

    const int cpt = a.C / BK;                      // chunks per filter tap
    const int nk = a.R * a.S * cpt;
    // Workgroups run in step, and chunk k of every pixel row and every weight row lies at the same offset inside rows whose
    // pitch is a large power of two: all requests of the moment fall on the same few offsets.  Each pixel tile therefore
    // starts the walk over the reduction at a chunk of its own (inside the first filter tap; the channel tiles of a pixel
    // tile share it) and wraps around: the same terms, summed in an order that depends on the tile index alone.  (The same
    // walk in the K-split, halo and whole-bottleneck kernels measured slower and is not used there.)
    const int rot = (tile / a.ntc) % cpt;
    int tr = 0, ts = 0, tcc = rot, tap = 0, tk = rot;   // filter tap / chunk of the NEXT stage to issue; tk: its index in the packed rows

    // the IDX-th DMA instruction of this wave for a stage; xsoff / wsoff: the stage's scalar offsets
    auto issue_one = [&](auto IDX, int buf, unsigned xsoff, unsigned wsoff, int tapbit) {
        constexpr int idx = decltype(IDX)::value;
        unsigned char *lx = lds + buf * STAGE, *lw = lx + BP * ROWB;
        if constexpr (idx < XL) {
            // sign-extended invalid-tap bit: all ones pushes the offset out of range -> zeros
            const unsigned off = xo[idx] | (unsigned)__builtin_amdgcn_sbfe(xinv[idx], tapbit, 1);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, (__attribute__((address_space(3))) void *)(lx + (wave * XL + idx) * 1024),
                                                     16, off, xsoff, 0, 0);
        } else {
            constexpr int wi = idx - XL;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(wr, (__attribute__((address_space(3))) void *)(lw + (wave * WL + wi) * 1024),
                                                     16, wo[wi], wsoff, 0, 0);
        }
    };
    auto x_soff = [&]() { return (unsigned)((tr * a.W + ts) * a.C + tcc * BK) * ES; };
    auto next_tap = [&]() {
        if (++tk == nk) { tk = 0; tcc = 0; tap = 0; ts = 0; tr = 0; return; }
        if (++tcc == cpt) { tcc = 0; ++tap; if (++ts == a.S) { ts = 0; ++tr; } }
    };
    auto issue = [&](int buf) {
        const unsigned xs = x_soff(), ws = (unsigned)(tk * BK) * ES;
        static_for<L>([&](auto IDX) { issue_one(IDX, buf, xs, ws, tap); });
        next_tap();
    };

    f32x16_t acc[TC][TP];
#pragma unroll
    for (int i = 0; i < TC; i++)
#pragma unroll
        for (int j = 0; j < TP; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

    const int lr = lane & 31, lh = lane >> 5;
    const int fsw = swz(lr);                       // tile row bases are multiples of 32: swizzle depends on lr only
    unsigned fx[KS], fw[KS];                       // LDS byte offsets of this lane's fragment rows, per k-step
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
        const unsigned so = ((2 * ks + lh) ^ fsw) << 4;
        fx[ks] = lds_addr(lds) + (wp * TP * 32 + lr) * ROWB + so;
        fw[ks] = lds_addr(lds) + BP * ROWB + (wc * TC * 32 + lr) * ROWB + so;
    }

#pragma unroll
    for (int s = 0; s < NS - 1; s++)
        if (s < nk) issue(s);

    // Epilogue operands behind the first DMAs: the compiler waits for the scale / shift loads where their two code
    // paths merge, and ahead of the DMAs that wait would put a whole memory round trip in front of the first tile
    // load.  Issued here they are the youngest entries of the in-order vmcnt queue, which only makes the first
    // iteration's wait stricter.
    const Affine8 aff = load_affine<TC>(a, lane, c0 + wc * TC * 32);
    ResidualRegs<T, TP, TC> resregs;
    prefetch_residual<T, TP, TC>(a, lane, p0 + wp * TP * 32, c0 + wc * TC * 32, LinearRows{a.P}, resregs);

    // fragments of one k-step; two sets alternate so that the reads of step s+1 fly under the MFMAs of step s
    u32x4_t fa[2][TC], fb[2][TP];
    auto read_frags = [&](auto SET, unsigned ax, unsigned aw) {
        constexpr int set = decltype(SET)::value;
        static_for<TC>([&](auto I) { lds_read16_async<decltype(I)::value * 32 * ROWB>(fa[set][decltype(I)::value], aw); });
        static_for<TP>([&](auto J) { lds_read16_async<decltype(J)::value * 32 * ROWB>(fb[set][decltype(J)::value], ax); });
    };

    for (int kc = 0; kc < nk; kc++) {
        // stage kc has landed once at most the (NS-2) stages issued after it are outstanding
        if (kc + NS - 2 < nk) wait_vmcnt<(NS - 2) * L>(); else wait_vmcnt<0>();
        __syncthreads();                           // ... for every wave; and stage kc-1 is no longer read
        const bool more = kc + NS - 1 < nk;        // a stage to prefetch during this iteration?
        const int nbuf = (kc + NS - 1) % NS, ntap = tap;
        const unsigned nxs = x_soff(), nws = (unsigned)(tk * BK) * ES;
        const unsigned sb = (kc % NS) * STAGE;
        read_frags(std::integral_constant<int, 0>{}, fx[0] + sb, fw[0] + sb);
        static_for<KS>([&](auto KSI) {
            constexpr int ks = decltype(KSI)::value, cur = ks & 1;
            if constexpr (ks + 1 < KS) {
                read_frags(std::integral_constant<int, cur ^ 1>{}, fx[ks + 1] + sb, fw[ks + 1] + sb);
                wait_lgkmcnt<TC + TP>();           // LDS returns in order: all but the newest TC+TP reads are done
            } else {
                wait_lgkmcnt<0>();
            }
            static_for<TC>([&](auto I) { landed(fa[cur][decltype(I)::value]); });
            static_for<TP>([&](auto J) { landed(fb[cur][decltype(J)::value]); });
            // this k-step's share of the next stage's DMA, one instruction behind each of the first MFMAs
            constexpr int dlo = ks * L / KS, dhi = (ks + 1) * L / KS;
            static_for<TC * TP>([&](auto Q) {
                constexpr int q = decltype(Q)::value, i = q / TP, j = q % TP;
                Mma<T>::run(acc[i][j], fa[cur][i], fb[cur][j]);
                if constexpr (dlo + q < dhi) {
                    if (more) issue_one(std::integral_constant<int, dlo + q>{}, nbuf, nxs, nws, ntap);
                }
                if constexpr (q == TC * TP - 1) {  // more DMA than MFMAs in this step: the rest follows
                    static_for<(dhi - dlo > TC * TP) ? dhi - dlo - TC * TP : 0>([&](auto E) {
                        if (more) issue_one(std::integral_constant<int, dlo + TC * TP + decltype(E)::value>{}, nbuf, nxs, nws, ntap);
                    });
                }
            });
        });
        if (more) next_tap();
    }
    __syncthreads();                               // every wave is done with the tiles: the ring becomes strips
    conv_epilogue_auto<T, TP, TC>(a, acc, reinterpret_cast<float *>(lds), wave, lane, p0 + wp * TP * 32, c0 + wc * TC * 32,
                             aff, LinearRows{a.P}, resregs);
#endif
}

template <typename T, int BP, int BC, int WP, int WC, int ROWB, int NS>
static sol_status launch_dma_cfg(ConvArgs a, hipStream_t st) {
    a.ntc = ceil_div(a.Cout, BC);
    a.ntiles = ceil_div(a.P, BP) * a.ntc;
    const int grid = ((a.ntiles + 7) / 8) * 8;
    const double xbytes = (double)a.N * a.H * a.W * a.C * sizeof(T), wbytes = (double)a.Cout * a.Kp * sizeof(T);
    a.cpx = (a.ntc % 8 == 0 && wbytes > xbytes && wbytes > 1.5 * 1048576) ? a.ntc / 8 : 0;
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
        case D_128x128_64x5: return launch_dma_cfg<T, 128, 128, 2, 2, 64, 5>(a, st);
        case D_64x64_128x4: return launch_dma_cfg<T, 64, 64, 2, 2, 128, 4>(a, st);
        case D_256x128_128x3: return launch_dma_cfg<T, 256, 128, 2, 2, 128, 3>(a, st);
        case D_256x128_64x4: return launch_dma_cfg<T, 256, 128, 2, 2, 64, 4>(a, st);
        case D_128x256_64x4: return launch_dma_cfg<T, 128, 256, 2, 2, 64, 4>(a, st);
        case D_64x64_64x8: return launch_dma_cfg<T, 64, 64, 2, 2, 64, 8>(a, st);
        default: SOL_FAIL(SOL_ERR_UNSUPPORTED, "unknown conv tile id %d", tile);
    }
}

// Row bytes the tile id needs (the reduction chunk must divide Cin); 0 = not a DMA tile id.
int dma_tile_row_bytes(int tile) {
    if (tile >= D_128x128_64x4 && tile <= D_64x128_64x4) return 64;
    if (tile == D_128x128_64x5) return 64;
    if (tile >= D_128x128_128x2 && tile <= D_256x128_128x3) return 128;
    if (tile >= D_256x128_64x4 && tile <= D_64x64_64x8) return 64;
    return 0;
}

sol_status launch_conv_dma(const ConvArgs &a, int dt, int tile, hipStream_t st) {
    if (dt == SOL_BF16) return launch_dma_typed<bf16_t>(a, tile, st);
    if (dt == SOL_F32) return launch_dma_typed<float>(a, tile, st);
    SOL_FAIL(SOL_ERR_DTYPE, "unknown dtype %d", dt);
}

}  // namespace sol

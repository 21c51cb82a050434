// Fused convolution (implicit GEMM over up to 32 filter taps, any stride / padding) as an eight-wave GEMM with an
// LDS-DMA ring (gfx950).
//
// Same GEMM view, operand layout in LDS (rows of ROWB bytes, 16-byte slots XOR-permuted on the global
// side) and epilogue as conv_dma.hip, but built for ONE workgroup of eight waves per CU instead of
// several four-wave workgroups:
//   * two waves per SIMD share one tile, so a tile row is fetched once for twice the MFMA work (the
//     vector-memory path delivers ~55 bytes per clock and CU, which a 128x128 tile per four waves
//     already saturates at the MFMA rate) and an LDS fragment read of one wave hides under the MFMAs
//     of the other (a single wave gets 32 bytes per clock from LDS, exactly its MFMA demand);
//   * optional K split inside the workgroup (KSPL): the waves of a group take alternate k-steps of
//     every stage and add their accumulators through LDS at the end.  This keeps 64x64 wave tiles
//     (1 KB of fragments per MFMA) for output tiles as small as 64x128, which is what layers with few
//     output pixels and a long reduction need to fill 256 CUs;
//   * the loop of the halo kernel: the barrier that publishes stage s+1 sits between two k-steps of
//     stage s, the last k-step already reads the next stage's first fragments, every DMA is issued
//     unconditionally (beyond the end through a size-0 buffer resource -> zeros), no branch inside.
#include "conv_common.h"

namespace sol {

// WP x WC x KSPL = 8 waves; TP x TC: 32x32 accumulator blocks per wave; ROWB: bytes of reduction per
// tile row and stage; NS: ring stages.
template <typename T, int WP, int WC, int KSPL, int TP, int TC, int ROWB, int NS>
__global__ void __launch_bounds__(512) conv_gemm8_kernel(const ConvArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)
    using namespace lds_pipe;
    constexpr int NW = 8, NG = WP * WC, ES = (int)sizeof(T), BK = ROWB / ES;
    constexpr int KS = ROWB / 32, NK = KS / KSPL;          // k-steps per stage, and per wave
    constexpr int BP = WP * TP * 32, BC = WC * TC * 32;
    constexpr int SLOTS = ROWB / 16, RSEG = 64 / SLOTS;     // 16-byte slots per row, rows per 1 KB DMA segment
    constexpr int XL = BP / RSEG / NW, WL = BC / RSEG / NW, L = XL + WL;
    constexpr int STAGE = (BP + BC) * ROWB, D = NS - 1;
    constexpr int BQ = NK / 2;                             // the publishing barrier precedes this k-step slot
    constexpr int ACCB = TC * TP * 16 * 64 * 4;            // bytes of one wave's accumulators
    constexpr int EPI0 = (KSPL - 1) * NG * ACCB;           // epilogue strips start behind the K-split partials
    static_assert(WP * WC * KSPL == NW && KS % KSPL == 0, "wave grid");
    static_assert(BP % (RSEG * NW) == 0 && BC % (RSEG * NW) == 0, "tile rows must split into whole DMA segments per wave");
    static_assert(NS >= 3 && NS * STAGE + NW * 256 <= 160 * 1024, "ring: the stage published by the mid-stage barrier was issued a whole stage earlier");
    static_assert(EPI0 + NG * 32 * (TC * 32 + 4) * 4 <= NS * STAGE, "K-split partials and epilogue strips must fit in the ring");
    static_assert((D - 1) * L < 64, "vmcnt");

    __shared__ __align__(1024) unsigned char lds[NS * STAGE];
    __shared__ __align__(256) unsigned char l2sink[NW * 256];   // write-only landing pad of the L2 warm-up loads

    // every kernel argument the prologue needs, fetched in one batch
    asm volatile("" ::"s"(a.x), "s"(a.w), "s"(a.scale), "s"(a.shift), "s"(a.res), "s"(a.y), "s"(a.P), "s"(a.C), "s"(a.Cout),
                 "s"(a.H), "s"(a.W), "s"(a.Kp), "s"(a.ntc), "s"(a.ntiles), "s"(a.act), "s"(a.dw.mul), "s"(a.dh.mul), "s"(a.sh), "s"(a.pool), "s"(a.R), "s"(a.S), "s"(a.ph));

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave % NG, kq = wave / NG;             // output sub-tile of the wave, and its share of the k-steps
    const int wp = grp % WP, wc = grp / WP;
    const int lr = lane & 31, lh = lane >> 5;
    const int lslot = lane % SLOTS, lrow = lane / SLOTS;

    // XCD-aware tile order (see conv_dma.hip): a contiguous run of tiles per XCD, or, when the weights are the
    // larger operand, a set of channel tiles per XCD
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

    // The activation resource starts `bias` bytes before the tensor so that the offset of a row's window origin
    // (which lies in the padding for border pixels) is never negative; only in-range taps are fetched through it.
    const unsigned bias = (unsigned)((a.ph * a.W + a.pw) * a.C) * ES;
    const unsigned xbytes = (unsigned)a.N * a.H * a.W * a.C * ES, wbytes = (unsigned)a.Cout * a.Kp * ES;
    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<unsigned char *>(static_cast<const unsigned char *>(a.x)) - bias, 0, (int)(xbytes + bias), 0x00020000);
    const __amdgpu_buffer_rsrc_t wr = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.w), 0, (int)wbytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t xnull = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.x), 0, 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t wnull = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.w), 0, 0, 0x00020000);

    {   // warm this XCD's L2 with the weights it will stream (with the channel split: only its channel tiles' rows)
        const unsigned slice = (unsigned)(a.cpx * BC * a.Kp) * ES, first = a.cpx > 0 ? min(wbytes, (unsigned)xcd * slice) : 0u;
        warm_l2(static_cast<const unsigned char *>(a.w) + first, a.cpx > 0 ? min(slice, wbytes - first) : wbytes, l2sink + wave * 256,
                tid, NW * 64);
    }

    // ---- DMA lane offsets (one 16-byte slot of XL pixel rows and WL weight rows per stage); bit t of xinv: filter
    // tap t of that row reads padding (its offset is pushed out of range, the hardware returns zeros)
    unsigned xo[XL], xinv[XL], wo[WL];
#pragma unroll
    for (int i = 0; i < XL; i++) {
        const int row = (wave * XL + i) * RSEG + lrow;
        const int m = p0 + row;
        int n, op, oq;
        decode_pixel(a, m, n, op, oq);
        const int ih0 = op * a.sh - a.ph, iw0 = oq * a.sw - a.pw;
        const unsigned off = (unsigned)(((n * a.H + ih0) * a.W + iw0) * a.C) * ES + bias + ((lslot ^ swz<ROWB>(row)) << 4);
        const int slo = max(0, -iw0), shi = min(a.S, a.W - iw0), rlo = max(0, -ih0), rhi = min(a.R, a.H - ih0);
        const unsigned cval = shi > slo ? (unsigned)((1ull << shi) - 1ull) & ~((1u << slo) - 1u) : 0u;
        unsigned val = 0;
        for (int r = 0; r < a.R; r++) val |= (r >= rlo && r < rhi) ? cval << (r * a.S) : 0u;
        xo[i] = m < a.P ? off : 0xffffffffu;
        xinv[i] = ~val;
    }
#pragma unroll
    for (int i = 0; i < WL; i++) {
        const int row = (wave * WL + i) * RSEG + lrow;
        const int co = c0 + row;
        wo[i] = co < a.Cout ? (unsigned)(co * a.Kp) * ES + ((lslot ^ swz<ROWB>(row)) << 4) : 0xffffffffu;
    }
    // IDX-th DMA instruction of this wave for a stage (pixel rows first); xsoff / wsoff: the stage's scalar byte offsets
    // (filter tap + reduction chunk), tapbit: its filter tap
    auto issue_one = [&](auto IDX, int buf, unsigned xsoff, unsigned wsoff, int tapbit, bool real) {
        constexpr int idx = decltype(IDX)::value;
        unsigned char *lx = lds + buf * STAGE, *lw = lx + BP * ROWB;
        if constexpr (idx < XL) {
            const unsigned off = xo[idx] | (unsigned)__builtin_amdgcn_sbfe(xinv[idx], tapbit, 1);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(real ? xr : xnull, (__attribute__((address_space(3))) void *)(lx + (wave * XL + idx) * 1024),
                                                     16, off, xsoff, 0, 0);
        } else {
            __builtin_amdgcn_raw_ptr_buffer_load_lds(real ? wr : wnull, (__attribute__((address_space(3))) void *)(lw + (wave * WL + idx - XL) * 1024),
                                                     16, wo[idx - XL], wsoff, 0, 0);
        }
    };
    // filter tap / chunk of the next stage to issue
    const int cpt = a.C / BK;
    int tr = 0, ts = 0, tcc = 0, tap = 0;
    auto x_soff = [&]() { return (unsigned)((tr * a.W + ts) * a.C + tcc * BK) * ES; };
    auto next_tap = [&]() { if (++tcc == cpt) { tcc = 0; ++tap; if (++ts == a.S) { ts = 0; ++tr; } } };

    const int nk = a.R * a.S * cpt;
    // ---- prologue: the first D stages, then (behind them) the epilogue operands
#pragma unroll
    for (int s = 0; s < D; s++) {
        const bool real = s < nk;
        const unsigned xs = x_soff();
        const int tb = tap;
        static_for<L>([&](auto I) { issue_one(I, s, xs, (unsigned)(s * ROWB), tb, real); });
        next_tap();
    }
    const Affine8 aff = load_affine<TC>(a, lane, c0 + wc * TC * 32);
    ResidualRegs<T, TP, TC> resregs;
    resregs.on = false;
    // With a four-way K split the accumulators of three partner waves pass through this wave's registers at the end:
    // no room to hold residual rows across the loop as well (they would be spilled to scratch memory and back); such
    // tiles fetch the residual in the epilogue.  The same holds for wave tiles of eight accumulator blocks.
    if constexpr (KSPL < 4 && TC * TP < 8) {
        if (kq == 0) prefetch_residual<T, TP, TC>(a, lane, p0 + wp * TP * 32, c0 + wc * TC * 32, LinearRows{a.P}, resregs);
    }

    f32x16_t acc[TC][TP];
#pragma unroll
    for (int i = 0; i < TC; i++)
#pragma unroll
        for (int j = 0; j < TP; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

    // fragment addresses of k-step 0 in stage buffer 0; k-step ks flips address bits 5.. (slot ^ 2*ks)
    const unsigned fsw = swz<ROWB>(lr);
    const unsigned fx0 = lds_addr(lds) + (wp * TP * 32 + lr) * ROWB + ((lh ^ fsw) << 4);
    const unsigned fw0 = lds_addr(lds) + BP * ROWB + (wc * TC * 32 + lr) * ROWB + ((lh ^ fsw) << 4);

    u32x4_t fa[2][TC], fb[2][TP];
    auto read_frags = [&](auto SET, auto Q, unsigned sb) {      // fragments of this wave's Q-th k-step of the stage at byte offset sb
        constexpr int set = decltype(SET)::value, q = decltype(Q)::value;
        const unsigned kx = (unsigned)((kq * NK + q) << 5);
        const unsigned aw = xor_add(fw0, kx, sb), ax = xor_add(fx0, kx, sb);
        static_for<TC>([&](auto I) { lds_read16<decltype(I)::value * 32 * ROWB>(fa[set][decltype(I)::value], aw); });
        static_for<TP>([&](auto J) { lds_read16<decltype(J)::value * 32 * ROWB>(fb[set][decltype(J)::value], ax); });
    };
    auto mfmas = [&](auto SET, auto &&between) {
        constexpr int set = decltype(SET)::value;
        static_for<TC>([&](auto I) { landed(fa[set][decltype(I)::value]); });
        static_for<TP>([&](auto J) { landed(fb[set][decltype(J)::value]); });
        static_for<TC * TP>([&](auto Q) {
            constexpr int q = decltype(Q)::value, i = q / TP, j = q % TP;
            Mma<T>::run(acc[i][j], fa[set][i], fb[set][j]);
            between(Q);
        });
    };
    auto nothing = [](auto) {};

    wait_vmcnt<0>();                                     // stage 0 (and the rest of the prologue) has landed
    __builtin_amdgcn_s_barrier();
    read_frags(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, 0u);

    unsigned sb = 0;                                     // byte offset of the current stage in the ring
    int ibuf = D % NS;                                   // ring slot of the next DMA
    unsigned isoff = (unsigned)(D * ROWB);               // its reduction-chunk offset
    // one stage; PAR: which fragment set holds the stage's first k-step (alternates per stage when NK is odd)
    auto stage = [&](auto PAR, int s) {
        constexpr int par = decltype(PAR)::value;
        const unsigned sbn = sb + STAGE == NS * STAGE ? 0u : sb + STAGE;
        const bool real = s + D < nk;
        static_for<NK>([&](auto Q) {
            constexpr int q = decltype(Q)::value, cur = (q + par) & 1;
            if constexpr (q == BQ) {
                // stage s+1 (issued D-1 stages ago) has landed once only the DMAs issued after it are outstanding
                wait_vmcnt<(D >= 2 ? (D - 2) * L : 0)>();
                __builtin_amdgcn_s_barrier();           // ... for every wave; and nobody still reads stage s-1
            }
            if constexpr (q + 1 < NK) read_frags(std::integral_constant<int, cur ^ 1>{}, std::integral_constant<int, q + 1>{}, sb);
            else read_frags(std::integral_constant<int, cur ^ 1>{}, std::integral_constant<int, 0>{}, sbn);
            wait_lgkmcnt<TC + TP>();
            if constexpr (q == BQ) {
                const int buf = ibuf, tb = tap;
                const unsigned so = isoff, xs = x_soff();
                mfmas(std::integral_constant<int, cur>{}, [&](auto M) {
                    constexpr int m = decltype(M)::value;
                    if constexpr (m < L) issue_one(M, buf, xs, so, tb, real);
                    if constexpr (m == TC * TP - 1)
                        static_for<(L > TC * TP) ? L - TC * TP : 0>([&](auto E) {
                            issue_one(std::integral_constant<int, TC * TP + decltype(E)::value>{}, buf, xs, so, tb, real);
                        });
                });
            } else {
                mfmas(std::integral_constant<int, cur>{}, nothing);
            }
        });
        ibuf = ibuf + 1 == NS ? 0 : ibuf + 1;
        isoff += ROWB;
        next_tap();
        sb = sbn;
    };
    if constexpr (NK % 2 == 0) {
        for (int s = 0; s < nk; s++) stage(std::integral_constant<int, 0>{}, s);
    } else {
        for (int s = 0; s < nk; s += 2) {
            stage(std::integral_constant<int, 0>{}, s);
            if (s + 1 < nk) stage(std::integral_constant<int, 1>{}, s + 1);
        }
    }
    wait_vmcnt<0>();
    wait_lgkmcnt<0>();
    __builtin_amdgcn_s_barrier();                        // the ring is dead: it becomes K-split partials and epilogue strips

    if constexpr (KSPL > 1) {
        // waves kq > 0 park their accumulators (lane-contiguous 16-byte pieces), wave kq == 0 of the group adds them
        float *part = reinterpret_cast<float *>(lds);
        if (kq > 0) {
            float *dst = part + ((size_t)((kq - 1) * NG + grp) * (ACCB / 4)) + lane * 4;
#pragma unroll
            for (int i = 0; i < TC; i++)
#pragma unroll
                for (int j = 0; j < TP; j++)
#pragma unroll
                    for (int g = 0; g < 4; g++)
                        *reinterpret_cast<float4 *>(dst + ((i * TP + j) * 4 + g) * 256) =
                            make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
        }
        __syncthreads();
        if (kq > 0) return;
#pragma unroll
        for (int k = 1; k < KSPL; k++) {
            const float *src = part + ((size_t)((k - 1) * NG + grp) * (ACCB / 4)) + lane * 4;
#pragma unroll
            for (int i = 0; i < TC; i++)
#pragma unroll
                for (int j = 0; j < TP; j++)
                {
#pragma unroll
                    for (int g = 0; g < 4; g++) {
                        const float4 v = *reinterpret_cast<const float4 *>(src + ((i * TP + j) * 4 + g) * 256);
                        acc[i][j][4 * g] += v.x; acc[i][j][4 * g + 1] += v.y; acc[i][j][4 * g + 2] += v.z; acc[i][j][4 * g + 3] += v.w;
                    }
                    asm volatile("" : "+v"(acc[i][j]) : : "memory");   // one accumulator block at a time (with every partner's loads hoisted the registers run out): the sums must exist here, later loads stay behind
                }
        }
    }
    conv_epilogue_auto<T, TP, TC>(a, acc, reinterpret_cast<float *>(lds + EPI0), grp, lane, p0 + wp * TP * 32, c0 + wc * TC * 32,
                                  aff, LinearRows{a.P}, resregs);
#endif
}

template <typename T, int WP, int WC, int KSPL, int TP, int TC, int ROWB, int NS>
static sol_status launch_gemm8_cfg(ConvArgs a, hipStream_t st) {
    constexpr int BP = WP * TP * 32, BC = WC * TC * 32;
    SOL_REQUIRE(a.C % (ROWB / (int)sizeof(T)) == 0, SOL_ERR_UNSUPPORTED, "conv tile needs Cin %% %d == 0", ROWB / (int)sizeof(T));
    a.ntc = ceil_div(a.Cout, BC);
    a.ntiles = ceil_div(a.P, BP) * a.ntc;
    const int grid = ((a.ntiles + 7) / 8) * 8;
    const double xbytes = (double)a.N * a.H * a.W * a.C * sizeof(T), wbytes = (double)a.Cout * a.Kp * sizeof(T);
    a.cpx = (a.ntc % 8 == 0 && wbytes > xbytes && wbytes > 1.5 * 1048576) ? a.ntc / 8 : 0;
    hipLaunchKernelGGL((conv_gemm8_kernel<T, WP, WC, KSPL, TP, TC, ROWB, NS>), dim3(grid), dim3(512), 0, st, a);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

// bf16, at most 32 filter taps (one validity bit each), Cin a multiple of 32, 32-bit byte offsets
bool gemm8_kernel_applies(const ConvArgs &a, int dt) {
    if (dt != SOL_BF16) return false;
    const double xb = (double)a.N * a.H * a.W * a.C * 2.0 + (double)(a.ph * a.W + a.pw) * a.C * 2.0, wb = (double)a.Cout * a.Kp * 2.0;
    return a.R * a.S <= 32 && a.C % 32 == 0 && xb < 4294967296.0 && wb < 4294967296.0;
}

sol_status launch_conv_gemm8(const ConvArgs &a, int tile, hipStream_t st) {
    switch (tile) {
        //                                              WP WC KSPL TP TC ROWB NS
        case G_128x128_k2: return launch_gemm8_cfg<bf16_t, 2, 2, 2, 2, 2, 128, 4>(a, st);
        case G_256x128: return launch_gemm8_cfg<bf16_t, 4, 2, 1, 2, 2, 128, 3>(a, st);
        case G_128x256: return launch_gemm8_cfg<bf16_t, 2, 4, 1, 2, 2, 128, 3>(a, st);
        case G_64x128_k4: return launch_gemm8_cfg<bf16_t, 1, 2, 4, 2, 2, 128, 5>(a, st);
        case G_128x64_k4: return launch_gemm8_cfg<bf16_t, 2, 1, 4, 2, 2, 128, 5>(a, st);
        case G_256x256_r64: return launch_gemm8_cfg<bf16_t, 2, 4, 1, 4, 2, 64, 4>(a, st);
        case G_256x128_r64: return launch_gemm8_cfg<bf16_t, 4, 2, 1, 2, 2, 64, 6>(a, st);
        case G_64x64_k4: return launch_gemm8_cfg<bf16_t, 2, 1, 4, 1, 2, 128, 6>(a, st);
        case G_64x64_k4_deep: return launch_gemm8_cfg<bf16_t, 2, 1, 4, 1, 2, 128, 9>(a, st);   // weight streaming: 8 stages in flight
        case G_64x32_k4_r256: return launch_gemm8_cfg<bf16_t, 2, 1, 4, 1, 1, 256, 6>(a, st);   // ... for matrices with < 200 tiles of 64 rows
        default: SOL_FAIL(SOL_ERR_UNSUPPORTED, "unknown gemm8 conv tile id %d", tile);
    }
}

}  // namespace sol

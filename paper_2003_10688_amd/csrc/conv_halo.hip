// Fused 3x3 / stride-1 / pad-1 convolution with the input halo staged once in LDS (gfx950).
//
// The implicit-GEMM kernels fetch every input pixel once per filter tap: nine trips through the
// vector-memory path (about 55 bytes per clock and CU, measured, against 128 bytes per clock that a
// 128x128 tile needs at the MFMA rate), which is what bounds them on 3x3 layers.  Here a workgroup
// owns BP *consecutive* output pixels (n, h, w flattened; output and input pixel indices coincide for
// stride 1 / pad 1) and BC output channels.  For one chunk of 64 input channels (one 128-byte row per
// pixel) it stages the input rows  [p0 - W - 1, p0 + BP + W + 1)  -- the tile and its halo -- in LDS
// once ("patch") and runs all nine taps from it: tap (r, s) of tile pixel m is patch row m + r*W + s.
// Taps that fall outside the image (they would read the neighbouring row / image in the flattened
// order) are redirected, per lane, to a row of zeros.  Only the weights still travel once per tap:
// a ring of NSW stages of BC x 128 bytes, one stage per (chunk, tap).
//
// Both operands go HBM/L2 -> LDS by DMA (buffer_load ... lds, 1 KB per wave instruction), 16-byte
// slots XOR-permuted with the row index on the global side so that the MFMA fragment reads are
// bank-conflict free.  Pipeline per stage (tap): k-steps 0,1 | wait for the DMA of the NEXT stage +
// workgroup barrier | issue the DMA D stages ahead | k-steps 2,3, the last of which already reads the
// next stage's first fragments.  The barrier therefore never separates a fragment read from its MFMAs,
// every DMA is issued unconditionally (beyond the end through a buffer resource of size 0, which the
// hardware turns into zeros) so that the in-order vmcnt bookkeeping is static, and there is no branch
// inside the loop.  Eight waves per workgroup (two per SIMD) keep the matrix cores fed while one wave
// waits.  With KSPL > 1 the waves of a group split the k-steps of every stage between them and add
// their accumulators through LDS at the end, which keeps 64x64 wave tiles for output tiles as small as
// 64x128 (layers with few output pixels and a long reduction).
#include "conv_common.h"

namespace sol {

// T: element type; WP x WC x KSPL: wave grid (pixels x channels x split of a stage's k-steps); TP x TC: 32x32
// accumulator blocks per wave; XL: patch DMA instructions per wave and chunk (patch rows = XL * waves * 8 >=
// BP + 2W + 2); NSW: weight ring stages; NPB: patch buffers (2, or 1 when Cin is a single chunk); MINW: waves per
// SIMD the register allocation must allow (4: two workgroups per CU).
template <typename T, int WP, int WC, int KSPL, int TP, int TC, int XL, int NSW, int NPB, int MINW = 2>
__global__ void __launch_bounds__(WP *WC *KSPL * 64, MINW) conv_halo_kernel(const ConvArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)
    using namespace lds_pipe;
    constexpr int NG = WP * WC, NW = NG * KSPL, ES = (int)sizeof(T), ROWB = 128, BK = ROWB / ES;
    constexpr int KS = ROWB / 32, NK = KS / KSPL;  // k-steps per stage, and per wave
    constexpr int BQ = NK / 2;                     // the publishing barrier precedes this k-step slot
    constexpr int BP = WP * TP * 32, BC = WC * TC * 32;
    constexpr int WSTAGE = BC * ROWB;              // bytes of one weight stage
    constexpr int WL = BC / 8 / NW;                // weight DMA instructions per wave and stage
    constexpr int D = NSW - 1;                     // stages a weight DMA is issued ahead of its use
    constexpr int PROWS = XL * NW * 8;             // patch rows fetched per chunk
    constexpr int PBYTES = PROWS * ROWB + 1024;    // patch buffer: rows, then a block whose first row stays zero
    constexpr int LDSB = NSW * WSTAGE + NPB * PBYTES;
    constexpr int ACCB = TC * TP * 16 * 64 * 4;    // bytes of one wave's accumulators
    constexpr int EPI0 = (KSPL - 1) * NG * ACCB;   // epilogue strips start behind the K-split partials
    static_assert(KS % KSPL == 0 && (NK % 2 == 0 || NK == 1), "k-step split");
    static_assert(BC % (8 * NW) == 0, "a weight stage must split into whole 1 KB segments per wave");
    static_assert(D >= 2 && D <= 8, "ring depth");
    static_assert(LDSB + NW * 256 <= 160 * 1024, "LDS");
    static_assert(EPI0 + NG * 32 * (TC * 32 + 4) * 4 <= LDSB, "K-split partials and epilogue strips must fit");
    static_assert(NPB == 1 || XL <= 6, "the patch of the next chunk is issued during taps 0..XL-1");

    __shared__ __align__(1024) unsigned char lds[LDSB];
    __shared__ __align__(256) unsigned char l2sink[NW * 256];   // write-only landing pad of the L2 warm-up loads

    // all kernel arguments the loop needs in scalar registers at once: fetched piecemeal, each batch would cost its
    // own round trip to the argument buffer
    asm volatile("" ::"s"(a.x), "s"(a.w), "s"(a.scale), "s"(a.shift), "s"(a.res), "s"(a.y), "s"(a.P), "s"(a.C), "s"(a.Cout),
                 "s"(a.H), "s"(a.W), "s"(a.Kp), "s"(a.ntc), "s"(a.ntiles), "s"(a.act), "s"(a.dw.mul), "s"(a.dh.mul));

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave % NG, kq = wave / NG;     // output sub-tile of the wave, and its share of the k-steps
    const int wp = grp % WP, wc = grp / WP;
    const int lr = lane & 31, lh = lane >> 5;
    const int lslot = lane & 7, lrow = lane >> 3;

    // XCD-aware tile order: every XCD (blockIdx & 7) takes a contiguous run of tiles, so neighbouring pixel
    // tiles (shared halo rows) and the channel tiles of a pixel tile meet in one L2.
    const int tile = (int)(blockIdx.x & 7) * ((a.ntiles + 7) >> 3) + (int)(blockIdx.x >> 3);
    if (tile >= a.ntiles) return;
    const int p0 = (tile / a.ntc) * BP, c0 = (tile % a.ntc) * BC;
    const int W = a.W;

    const unsigned xbytes = (unsigned)a.P * a.C * ES, wbytes = (unsigned)a.Cout * a.Kp * ES;
    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.x), 0, (int)xbytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t wr = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.w), 0, (int)wbytes, 0x00020000);
    // size 0: every lane is out of range, the DMA writes zeros (used for the stages beyond the end)
    const __amdgpu_buffer_rsrc_t xnull = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.x), 0, 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t wnull = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.w), 0, 0, 0x00020000);

    unsigned char *const wring = lds, *const patch = lds + NSW * WSTAGE;
    warm_l2(static_cast<const unsigned char *>(a.w), wbytes, l2sink + wave * 256, tid, NW * 64);

    // ---- DMA lane offsets: XL patch segments and WL weight segments per wave, 8 rows x 8 slots each
    unsigned xo[XL], wo[WL];
#pragma unroll
    for (int i = 0; i < XL; i++) {
        const int row = (wave + NW * i) * 8 + lrow;
        const int pin = p0 - W - 1 + row;
        xo[i] = (pin >= 0 && pin < a.P) ? (unsigned)pin * (unsigned)(a.C * ES) + ((lslot ^ swz<ROWB>(row)) << 4) : 0xffffffffu;
    }
#pragma unroll
    for (int i = 0; i < WL; i++) {
        const int row = (wave * WL + i) * 8 + lrow;
        const int co = c0 + row;
        wo[i] = co < a.Cout ? (unsigned)co * (unsigned)(a.Kp * ES) + ((lslot ^ swz<ROWB>(row)) << 4) : 0xffffffffu;
    }
    auto issue_patch = [&](auto I, int buf, unsigned soff, bool real) {
        constexpr int i = decltype(I)::value;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(real ? xr : xnull,
                                                 (__attribute__((address_space(3))) void *)(patch + buf * PBYTES + (wave + NW * i) * 1024),
                                                 16, xo[i], soff, 0, 0);
    };
    auto issue_w = [&](auto I, int slot, unsigned soff, bool real) {
        constexpr int i = decltype(I)::value;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(real ? wr : wnull,
                                                 (__attribute__((address_space(3))) void *)(wring + slot * WSTAGE + (wave * WL + i) * 1024),
                                                 16, wo[i], soff, 0, 0);
    };

    const unsigned fw0 = lds_addr(wring) + (wc * TC * 32 + lr) * ROWB + ((lh ^ swz<ROWB>(lr)) << 4);

    f32x16_t acc[TC][TP];
#pragma unroll
    for (int i = 0; i < TC; i++)
#pragma unroll
        for (int j = 0; j < TP; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

    const int nchunks = a.C / BK;
    const unsigned tapstride = (unsigned)(a.C * ES);     // bytes between the taps of a packed weight row

    // ---- prologue: patch of chunk 0 and the first D weight stages
    static_for<XL>([&](auto I) { issue_patch(I, 0, 0u, true); });
#pragma unroll
    for (int s = 0; s < D; s++) {
        const bool real = s < 9 * nchunks;             // always true for s < 9
        static_for<WL>([&](auto I) { issue_w(I, s, (unsigned)s * tapstride, real); });
    }
    // epilogue operands (scale / shift, residual rows) and the zero rows, all behind the first DMAs
    // (absent scale / shift -- the training forward stores the bare convolution -- read as 1 / 0)
    const Affine8 aff = (a.scale && a.shift) ? load_affine_unconditional<TC>(a, lane, c0 + wc * TC * 32) : load_affine<TC>(a, lane, c0 + wc * TC * 32);
    ResidualRegs<T, TP, TC> resregs;
    resregs.on = false;                                  // tight register budgets fetch residual rows in the epilogue instead
    if constexpr (MINW < 4 && KSPL < 4) {          // a four-way K split needs the registers for its partners' accumulators
        if (kq == 0) prefetch_residual<T, TP, TC>(a, lane, p0 + wp * TP * 32, c0 + wc * TC * 32, LinearRows{a.P}, resregs);
    }
    if (tid < NPB * 64) *reinterpret_cast<unsigned *>(patch + (tid >> 6) * PBYTES + PROWS * ROWB + (tid & 63) * 4) = 0u;   // two zero rows

    // ---- fragment addresses (computed while the first DMAs are in flight).  ax[j][t]: LDS byte address (patch
    // buffer 0, k-step 0) of tap t of this lane's pixel in pixel block j, or of the zero row when that tap lies
    // outside the image.  The k-step flips address bits 5-6 (slot ^ 2*ks), the patch buffer adds a multiple of 1 KB.
    unsigned ax[TP][9];
#pragma unroll
    for (int j = 0; j < TP; j++) {
        const int mloc = (wp * TP + j) * 32 + lr, m = p0 + mloc;
        int n, h, w;
        decode_pixel(a, m, n, h, w);                   // rows beyond the tensor decode to something; `inside` masks them
        const unsigned inside = m < a.P ? 1u : 0u;
        const unsigned hok[3] = {inside & (h >= 1 ? 1u : 0u), inside, inside & (h + 1 < a.H ? 1u : 0u)};
        const unsigned wok[3] = {w >= 1 ? 1u : 0u, 1u, w + 1 < W ? 1u : 0u};
        const unsigned zero_base = lds_addr(patch) + PROWS * ROWB;   // 256 zero bytes = one pass over all 64 banks
#pragma unroll
        for (int t = 0; t < 9; t++) {
            const int r = t / 3, sx = t % 3;
            const int row = mloc + r * W + sx;
            const unsigned real = lds_addr(patch) + row * ROWB + ((lh ^ swz<ROWB>(row)) << 4);
            // A redirected lane reads the zero bytes that lie in the banks of the patch slot it would have read (same
            // offset within a 256-byte bank pass), so a redirect never adds a bank conflict to the wave's read.
            const unsigned zero_row = zero_base + (real & 255u);
            // arithmetic select (no divergent branch): zero_row + ok * (real - zero_row)
            ax[j][t] = zero_row + ((0u - (hok[r] & wok[sx])) & (real - zero_row));
        }
    }
    wait_vmcnt<0>();                                     // patch 0, the first weight stages and the epilogue operands have landed
    __builtin_amdgcn_s_barrier();                        // ... everyone's; the zero rows are written

    u32x4_t fa[2][TC], fb[2][TP];
    // fragments of this wave's Q-th k-step of a stage: tap TAP, weight ring offset wsoff, patch buffer offset pboff
    auto read_frags = [&](auto SET, auto TAP, auto Q, unsigned wsoff, unsigned pboff) {
        constexpr int set = decltype(SET)::value, t = decltype(TAP)::value, q = decltype(Q)::value;
        const unsigned kx = (unsigned)((kq * NK + q) << 5);
        const unsigned aw = xor_add(fw0, kx, wsoff);
        static_for<TC>([&](auto I) { lds_read16<decltype(I)::value * 32 * ROWB>(fa[set][decltype(I)::value], aw); });
        static_for<TP>([&](auto J) {
            constexpr int j = decltype(J)::value;
            lds_read16<0>(fb[set][j], xor_add(ax[j][t], kx, pboff));
        });
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
    using I0 = std::integral_constant<int, 0>;

    read_frags(I0{}, I0{}, I0{}, 0u, 0u);

    unsigned wsoff = 0;                                  // ring slot (bytes) of the current stage
    int islot = D % NSW;                                 // ring slot the next weight DMA goes to
    // one chunk of input channels = nine stages; PAR: which fragment set holds the chunk's first k-step (the sets
    // alternate per k-step, so with an odd number of k-steps per chunk it alternates per chunk)
    auto chunk = [&](auto PAR, int c) {
        constexpr int par = decltype(PAR)::value;
        const unsigned pboff = NPB == 2 ? (unsigned)(c & 1) * PBYTES : 0u;
        const unsigned pbnext = NPB == 2 ? (unsigned)((c + 1) & 1) * PBYTES : 0u;
        const bool more_chunks = c + 1 < nchunks;
        static_for<9>([&](auto TAP) {
            constexpr int t = decltype(TAP)::value;
            constexpr int tn = (t + 1) % 9;             // tap of the next stage
            constexpr int ti = (t + D) % 9, ci = (t + D) / 9;   // tap / chunk increment of the stage whose DMA is issued
            const unsigned wsnext = wsoff + WSTAGE == NSW * WSTAGE ? 0u : wsoff + WSTAGE;
            static_for<NK>([&](auto Q) {
                constexpr int q = decltype(Q)::value, cur = (par + t * NK + q) & 1;
                if constexpr (q == BQ) {
                    // The next stage's weights (issued D-1 stages ago) have landed once only the DMAs issued after
                    // them are outstanding: per stage WL weight instructions, then one patch instruction in taps 0..XL-1.
                    // (The stages issued since are s+2 .. s+D-1, issued during stages s-D+2 .. s-1; the patch instruction of
                    // stage s-D+1 follows that stage's weights, i.e. the ones being waited for, so it counts as well.)
                    constexpr int NPATCH = [] { int n = 0; for (int k = 1; k <= D - 1; k++) n += (NPB == 2 && t - k >= 0 && t - k < XL) ? 1 : 0; return n; }();
                    // Before the last tap's barrier the next chunk's patch (last instruction issued in tap XL-1) must have
                    // landed too: then at most the weights issued in taps XL..7 may be outstanding.
                    constexpr int GEN = (D - 2) * WL + NPATCH, LASTTAP = (8 - XL) * WL;
                    wait_vmcnt<(t == 8 && NPB == 2 && LASTTAP < GEN) ? LASTTAP : GEN>();
                    __builtin_amdgcn_s_barrier();       // ... for every wave; and nobody still reads stage s-1 / the other patch
                }
                // fragments of the next k-step: of this stage, or (published by the barrier) the next stage's first
                if constexpr (q + 1 < NK) read_frags(std::integral_constant<int, cur ^ 1>{}, TAP, std::integral_constant<int, q + 1>{}, wsoff, pboff);
                else read_frags(std::integral_constant<int, cur ^ 1>{}, std::integral_constant<int, tn>{}, I0{}, wsnext, t == 8 ? pbnext : pboff);
                wait_lgkmcnt<TC + TP>();
                if constexpr (q == BQ) {
                    const bool wreal = ci == 0 ? true : (c + ci < nchunks);
                    const unsigned wsoffg = (unsigned)ti * tapstride + (unsigned)((c + ci) * ROWB);
                    const int slot = islot;
                    mfmas(std::integral_constant<int, cur>{}, [&](auto M) {
                        constexpr int m = decltype(M)::value;
                        if constexpr (m < WL) issue_w(M, slot, wsoffg, wreal);
                        if constexpr (m == TC * TP - 1) {
                            static_for<(WL > TC * TP) ? WL - TC * TP : 0>([&](auto E) {
                                issue_w(std::integral_constant<int, TC * TP + decltype(E)::value>{}, slot, wsoffg, wreal);
                            });
                            if constexpr (NPB == 2 && t < XL) issue_patch(TAP, (c + 1) & 1, (unsigned)((c + 1) * ROWB), more_chunks);
                        }
                    });
                } else {
                    mfmas(std::integral_constant<int, cur>{}, nothing);
                }
            });
            islot = islot + 1 == NSW ? 0 : islot + 1;
            wsoff = wsnext;
        });
    };
    if constexpr (NK % 2 == 0) {
        for (int c = 0; c < nchunks; c++) chunk(I0{}, c);
    } else {
        for (int c = 0; c < nchunks; c += 2) {
            chunk(I0{}, c);
            if (c + 1 < nchunks) chunk(std::integral_constant<int, 1>{}, c + 1);
        }
    }
    wait_vmcnt<0>();                                     // the zero-fill DMAs of the tail
    wait_lgkmcnt<0>();
    __builtin_amdgcn_s_barrier();                        // every wave is done with the ring: it becomes partials and strips

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

template <typename T, int WP, int WC, int KSPL, int TP, int TC, int XL, int NSW, int NPB, int MINW = 2>
static sol_status launch_halo_cfg(ConvArgs a, hipStream_t st) {
    constexpr int BP = WP * TP * 32, BC = WC * TC * 32, PROWS = XL * WP * WC * KSPL * 8;
    SOL_REQUIRE(BP + 2 * a.W + 2 <= PROWS, SOL_ERR_UNSUPPORTED, "halo tile: image width %d needs %d patch rows, tile has %d", a.W,
                BP + 2 * a.W + 2, PROWS);
    SOL_REQUIRE(NPB == 2 || a.C * (int)sizeof(T) == 128, SOL_ERR_UNSUPPORTED, "single patch buffer needs Cin = one 128-byte chunk");
    a.ntc = ceil_div(a.Cout, BC);
    a.ntiles = ceil_div(a.P, BP) * a.ntc;
    const int grid = ((a.ntiles + 7) / 8) * 8;
    hipLaunchKernelGGL((conv_halo_kernel<T, WP, WC, KSPL, TP, TC, XL, NSW, NPB, MINW>), dim3(grid), dim3(WP * WC * KSPL * 64), 0, st, a);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

// 3x3, stride 1, pad 1, no fused pool, Cin a multiple of the 128-byte chunk, 32-bit byte offsets with headroom
// (offsets of rows before the tensor wrap to values above its size).
bool halo_kernel_applies(const ConvArgs &a, int dt) {
    if (dt != SOL_BF16) return false;
    const double xb = (double)a.P * a.C * 2.0, wb = (double)a.Cout * a.Kp * 2.0;
    return a.R == 3 && a.S == 3 && a.sh == 1 && a.sw == 1 && a.ph == 1 && a.pw == 1 && a.pool == 0 && a.C % 64 == 0 &&
           a.Cout % 8 == 0 && a.Ho == a.H && a.Wo == a.W && a.W <= 62 && xb < 2147483648.0 && wb < 2147483648.0;
}

// Shape heuristic (sol_network_autotune refines it by timing): one workgroup per CU wants about 200 tiles or
// several rounds of them.
int halo_choose_tile(const ConvArgs &a) {
    const bool single = a.C == 64;
    if (a.Cout <= 64) return a.W <= 30 ? H_256x64_x5 : (single ? H_256x64_x6s2 : H_256x64_x6);
    if (a.W > 30) return 0;
    const long nt256 = (long)ceil_div(a.P, 256) * ceil_div(a.Cout, 128);
    if (nt256 >= 160) return H_256x128_x5;
    if (nt256 >= 80) return H_128x128_k2;
    return H_64x128_k4;
}

sol_status launch_conv_halo(const ConvArgs &a, int tile, hipStream_t st) {
    switch (tile) {
        //                                                WP WC KSPL TP TC XL NSW NPB MINW
        case H_256x128_x5: return launch_halo_cfg<bf16_t, 4, 2, 1, 2, 2, 5, 4, 2>(a, st);
        case H_128x128_x3: return launch_halo_cfg<bf16_t, 2, 4, 1, 2, 1, 3, 4, 2>(a, st);
        case H_256x64_x5: return launch_halo_cfg<bf16_t, 4, 2, 1, 2, 1, 5, 4, 2>(a, st);
        case H_256x64_x6s: return launch_halo_cfg<bf16_t, 4, 2, 1, 2, 1, 6, 4, 1>(a, st);
        case H_256x64_x6s2: return launch_halo_cfg<bf16_t, 4, 2, 1, 2, 1, 6, 3, 1, 4>(a, st);   // 74 KB, <= 128 VGPRs: two workgroups per CU
        case H_256x64_x6: return launch_halo_cfg<bf16_t, 4, 2, 1, 2, 1, 6, 4, 2>(a, st);          // wide images (up to 62 columns), several chunks of input channels
        case H_128x128_k2: return launch_halo_cfg<bf16_t, 2, 2, 2, 2, 2, 3, 4, 2>(a, st);
        case H_64x128_k4: return launch_halo_cfg<bf16_t, 1, 2, 4, 2, 2, 2, 5, 2>(a, st);
        case H_128x64_k4: return launch_halo_cfg<bf16_t, 2, 1, 4, 2, 2, 3, 8, 2>(a, st);
        case H_64x64_k4: return launch_halo_cfg<bf16_t, 1, 1, 4, 2, 2, 4, 5, 2>(a, st);   // four waves, 75 KB: two workgroups per CU
        default: SOL_FAIL(SOL_ERR_UNSUPPORTED, "unknown halo conv tile id %d", tile);
    }
}

}  // namespace sol

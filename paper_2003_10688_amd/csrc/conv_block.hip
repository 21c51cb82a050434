// A whole residual bottleneck -- 1x1 reduce, 3x3, 1x1 expand, each with folded BN, the identity shortcut and the
// ReLUs -- as ONE depth-first kernel (gfx950, bf16):
//
//     t1 = relu(s1 * (x  . W1) + h1)          [P][WM]     1x1, C4 -> WM channels
//     t2 = relu(s2 * (t1 * W2) + h2)          [P][WM]     3x3, stride 1, pad 1
//     y  = relu(s3 * (t2 . W3) + h3 + x)      [P][C4]     1x1, WM -> C4 channels, shortcut = the block input
//
// This is the paper's depth-first processing (Sec. III-A: a chain of layers is run over a block of data while it
// sits in registers and on-chip memory) applied across the contractions.  Run layer by layer, t1 and t2 are
// written to and read from HBM and x is read twice; here a workgroup owns `bp` consecutive output pixels
// (n, h, w flattened), and per tile
//   A  computes t1 for the tile and its halo (the rows [p0 - W - 1, p0 + bp + W + 1): everything a 3x3 window of
//      a tile pixel can touch) from x streamed through an LDS ring in slices of 32 channels, and parks it in LDS as
//      bf16 -- the same rounding point as the stored tensor of the layer-by-layer path;
//   B  runs the nine taps of the 3x3 from that patch (tap (r, s) of tile pixel m = patch row m + r*W + s; taps
//      outside the image are redirected per lane to a row of zeros), only the weights travel, and parks t2 in LDS;
//   C  contracts t2 with W3 in passes of 128 output channels and stores y through the shared epilogue, the
//      shortcut rows of x prefetched into registers.
// HBM sees x once (plus the halo rows, which neighbouring tiles share through L2), the weights, and y.
// All three phases use one pipeline: operands reach LDS by DMA (buffer_load ... lds) into a ring of NS slots, one
// workgroup barrier per stage, fragment reads as opaque statements ordered by hand (the compiler would make every
// LDS read wait for all outstanding DMA), every DMA issued unconditionally (beyond the end through a size-0 buffer
// resource) so that the in-order vmcnt bookkeeping is static.  The first stages of the next phase are issued before
// the epilogue of the current one, which therefore writes LDS with bare ds_write statements.
#include <algorithm>

#include "conv_common.h"

namespace sol {

struct BlockArgs {
    const void *x;
    void *y;
    const void *w1, *w2, *w3;                        // packed [WM][C4], [WM][9*WM] (tap-major), [C4][WM]
    const float *s1, *h1, *s2, *h2, *s3, *h3;        // folded BN + bias of the three convolutions (scale, shift)
    int P, H, W, C4;                                 // pixels N*H*W, image extent, block channels
    int bp;                                          // output pixels per tile
    int ntiles;
    FastDiv dw, dh;                                  // by W, by H
};

// NW: waves per workgroup (8: one workgroup per CU.  A four-wave configuration with 128-pixel tiles and two workgroups
// per CU -- <4, 64, 256, 4, 2, 4, 2, 2, 1, 3, 4>, 68 KB of LDS -- gives the same results and the same time on the 56x56
// blocks, 80.9 against 81.2 us: the kernel is bound by the bytes that cross the fabric, not by latency); WM: mid channels (64 or 128); PRA: patch rows held in LDS (>= bp + 2W + 2, a multiple of 16); NBO: 32-pixel blocks
// of a tile (bp <= 32 NBO); wave grids (pixels x channels, product 8) and 32x32 accumulator blocks per wave for the
// phases A and B (C follows from WM: passes of 128 channels on 2 x 4 waves for WM = 64, of 64 channels on 4 x 2 waves
// for WM = 128, one 32-channel block per wave); ring depths of A and B.
template <int NW, int WM, int PRA, int NBO, int WPA, int TPA, int WPB, int TPB, int TCB, int NSA, int NSB>
__global__ void __launch_bounds__(NW * 64, 512 / (NW * 64)) conv_block_kernel(const BlockArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)
    using namespace lds_pipe;
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    constexpr int CH = WM / 64;                                       // 64-channel planes of t1 / t2
    constexpr int WCA = NW / WPA, TCA = WM / 32 / WCA;
    constexpr int WCB = NW / WPB;
    constexpr int PC = WM == 64 ? 128 : 64;                          // output channels per pass of phase C: PC * WM * 2 = 16 KB of W3
    constexpr int WCC = PC / 32, WPC = NW / WCC, TPC = NBO / WPC;
    static_assert(WM % 64 == 0 && TCA == 1 && WPA * TPA * 32 >= PRA && PRA % 16 == 0, "phase A tiling");
    static_assert(WPB * TPB == NBO && WCB * TCB * 32 == WM, "phase B tiling");
    static_assert(NBO % WPC == 0, "phase C tiling");
    // LDS map (overlaid: the phases never need everything at once)
    //   phase A:  [ring of NSA slots ...........................................]            (t1 is written after the loop)
    //   phase B:  [t1 planes: rows, zero block          ][ring of NSB weight slots]
    //   phase C:  [t2 planes            ][two W3 buffers][epilogue strips]
    constexpr int PLANE1 = PRA * 128 + 256, PLANE2 = NBO * 32 * 128;
    constexpr int R0 = (CH * PLANE1 > CH * PLANE2 ? CH * PLANE1 : CH * PLANE2);
    constexpr int XROWB = 64;                                         // phase A: bytes of reduction per row and stage
    constexpr int SLOTA = (PRA + WM) * XROWB, SLOTB = WM * 128, PCBUF = PC * WM * 2;
    constexpr int STRIPS = NW * 32 * (32 + 4) * 4;
    constexpr int LB_ = R0 + NSB * SLOTB, LC_ = CH * PLANE2 + 2 * PCBUF + STRIPS;
    constexpr int LBC = LB_ > LC_ ? LB_ : LC_;
    constexpr int LMAIN = NSA * SLOTA > LBC ? NSA * SLOTA : LBC;
    constexpr int LDSB = LMAIN + 1024;
    static_assert(LDSB <= 160 * 1024, "LDS");
    static_assert(R0 % 256 == 0 && PCBUF == 16384, "alignment of the ring area; one pass of W3 is sixteen 1 KB DMA segments");
    static_assert(NW == 8 || NW == 4, "one or two workgroups per CU");
    // DMA instructions per wave and stage
    constexpr int NXI = PRA / 16, XLA = (NXI + NW - 1) / NW, NWIA = WM / 16, WLA = (NWIA + NW - 1) / NW, LA = XLA + WLA;
    constexpr int LB = WM / 8 / NW, LC = PCBUF / 1024 / NW;
    static_assert(LB >= 1 && LC >= 1 && (NSA - 1) * LA < 64 && (NSB - 1) * LB < 64, "vmcnt");

    __shared__ __align__(1024) unsigned char lds[LDSB];
    unsigned char *const t1 = lds, *const ringA = lds, *const ring = lds + R0, *const ringC = lds + CH * PLANE2, *const dump = lds + LMAIN;

    asm volatile("" ::"s"(a.x), "s"(a.y), "s"(a.w1), "s"(a.w2), "s"(a.w3), "s"(a.s1), "s"(a.h1), "s"(a.s2), "s"(a.h2), "s"(a.s3),
                 "s"(a.h3), "s"(a.P), "s"(a.H), "s"(a.W), "s"(a.C4), "s"(a.bp), "s"(a.ntiles), "s"(a.dw.mul), "s"(a.dh.mul));

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lr = lane & 31, lh = lane >> 5;
    const int tile = (int)(blockIdx.x & 7) * ((a.ntiles + 7) >> 3) + (int)(blockIdx.x >> 3);   // a contiguous run of tiles per XCD
    if (tile >= a.ntiles) return;
    const int W = a.W, C4 = a.C4;
    const int p0 = tile * a.bp, pend = min(p0 + a.bp, a.P);           // output pixels [p0, pend)
    const int pr = a.bp + 2 * W + 2;                                  // patch rows in use

    const unsigned xbytes = (unsigned)a.P * (unsigned)C4 * 2u;
    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.x), 0, (int)xbytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t w1r = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.w1), 0, WM * C4 * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t w2r = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.w2), 0, WM * 9 * WM * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t w3r = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.w3), 0, C4 * WM * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t nullr = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.x), 0, 0, 0x00020000);   // size 0: zeros

    // the weights are cold when the block starts: touch one dword per 128-byte line, spread over the XCD's workgroups
    warm_l2(static_cast<const unsigned char *>(a.w1), (unsigned)(WM * C4 * 2), dump + (wave & 3) * 256, tid, NW * 64);
    warm_l2(static_cast<const unsigned char *>(a.w2), (unsigned)(WM * 9 * WM * 2), dump + (wave & 3) * 256, tid, NW * 64);
    warm_l2(static_cast<const unsigned char *>(a.w3), (unsigned)(C4 * WM * 2), dump + (wave & 3) * 256, tid, NW * 64);

    // ---- DMA lane offsets of all three phases (a few registers each), so that a phase's first stages can be issued
    // before the epilogue of the phase in front of it
    // phase A, rows of 64 bytes: one instruction = 16 rows x 4 slots of 16 bytes
    unsigned xoA[XLA], woA[WLA];
    {
        const int lslot = lane & 3, lrow = lane >> 2;
#pragma unroll
        for (int i = 0; i < XLA; i++) {
            const int idx = wave + NW * i, row = idx * 16 + lrow;
            const int pin = p0 - W - 1 + row;
            const bool ok = idx < NXI && row < pr && pin >= 0 && pin < a.P;
            xoA[i] = ok ? (unsigned)pin * (unsigned)(C4 * 2) + (unsigned)((lslot ^ swz<XROWB>(row)) << 4) : 0xffffffffu;
        }
#pragma unroll
        for (int i = 0; i < WLA; i++) {
            const int idx = wave + NW * i, row = idx * 16 + lrow;
            woA[i] = idx < NWIA ? (unsigned)row * (unsigned)(C4 * 2) + (unsigned)((lslot ^ swz<XROWB>(row)) << 4) : 0xffffffffu;
        }
    }
    // phases B and C, rows of 128 bytes: one instruction = 8 rows x 8 slots
    unsigned woB[LB], woC[LC];
    {
        const int lslot = lane & 7, lrow = lane >> 3;
#pragma unroll
        for (int i = 0; i < LB; i++) {
            const int row = (wave * LB + i) * 8 + lrow;
            woB[i] = (unsigned)row * (unsigned)(9 * WM * 2) + (unsigned)((lslot ^ swz<128>(row)) << 4);
        }
#pragma unroll
        for (int i = 0; i < LC; i++) {
            const int idx = wave * LC + i, c = idx / (PC / 8), row = (idx % (PC / 8)) * 8 + lrow;   // plane c, row of the pass
            woC[i] = (unsigned)row * (unsigned)(WM * 2) + (unsigned)(c * 128) + (unsigned)((lslot ^ swz<128>(row)) << 4);
        }
    }
    auto issueA = [&](int slot, unsigned soff, bool real) {
        unsigned char *base = ringA + slot * SLOTA;
        static_for<XLA>([&](auto I) {
            constexpr int i = decltype(I)::value;
            const int idx = wave + NW * i;
            unsigned char *dst = idx < NXI ? base + idx * 1024 : dump;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(real ? xr : nullr, (__attribute__((address_space(3))) void *)dst, 16, xoA[i], soff, 0, 0);
        });
        static_for<WLA>([&](auto I) {
            constexpr int i = decltype(I)::value;
            const int idx = wave + NW * i;
            unsigned char *dst = idx < NWIA ? base + PRA * XROWB + idx * 1024 : dump;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(real ? w1r : nullr, (__attribute__((address_space(3))) void *)dst, 16, woA[i], soff, 0, 0);
        });
    };
    constexpr int nB = 9 * CH;
    auto issueB = [&](int slot, int sidx, bool real) {      // stage sidx = chunk * 9 + tap
        const int c = sidx / 9, tp = sidx - 9 * c;
        const unsigned soff = (unsigned)((tp * WM + c * 64) * 2);
        static_for<LB>([&](auto I) {
            constexpr int i = decltype(I)::value;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(real ? w2r : nullr,
                                                     (__attribute__((address_space(3))) void *)(ring + slot * SLOTB + (wave * LB + i) * 1024), 16,
                                                     woB[i], soff, 0, 0);
        });
    };
    const int npass = C4 / PC;
    auto issueC = [&](int buf, int q, bool real) {
        const unsigned soff = (unsigned)(q * PC * WM * 2);
        static_for<LC>([&](auto I) {
            constexpr int i = decltype(I)::value;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(real ? w3r : nullr,
                                                     (__attribute__((address_space(3))) void *)(ringC + buf * PCBUF + (wave * LC + i) * 1024), 16,
                                                     woC[i], soff, 0, 0);
        });
    };
    // BN + ReLU of a lane's four channels of one accumulator group, packed to bf16, stored at its place in a t1 / t2 plane
    // (row r, channel ch: plane ch / 64, 16-byte slot (ch % 64) / 8 permuted with the row, as the fragment reads expect).
    // A bare ds_write: a store the compiler knows of would wait for the next phase's DMAs, which are already in flight.
    auto park = [&](const f32x16_t &acc, int g, const float4 &sc, const float4 &sh, unsigned plane_bytes, int row, int ch) {
        float v0 = acc[4 * g] * sc.x + sh.x, v1 = acc[4 * g + 1] * sc.y + sh.y, v2 = acc[4 * g + 2] * sc.z + sh.z, v3 = acc[4 * g + 3] * sc.w + sh.w;
        v0 = __builtin_fmaxf(v0, 0.f); v1 = __builtin_fmaxf(v1, 0.f); v2 = __builtin_fmaxf(v2, 0.f); v3 = __builtin_fmaxf(v3, 0.f);   // one v_max each; a NaN becomes 0
        const unsigned long long pk = (unsigned long long)pack_bf16x2(v0, v1) | ((unsigned long long)pack_bf16x2(v2, v3) << 32);
        const unsigned dst = lds_addr(t1) + (unsigned)(ch >> 6) * plane_bytes + (unsigned)(row * 128) +
                             (unsigned)((((ch & 63) >> 3) ^ swz<128>(row)) << 4) + (unsigned)((ch & 7) * 2);
        asm volatile("ds_write_b64 %0, %1" ::"v"(dst), "v"(pk) : "memory");
    };

    // ================================================================ phase A: t1 = relu(bn1(x . W1)) over the patch rows
    const int nA = C4 / 32;
    // per-lane BN constants of phase A (16 channels: 4 groups of 4), loaded ahead of the DMAs: older loads never
    // disturb the static counts of the ring
    const int wpA = wave % WPA, wcA = wave / WPA;
    float4 scA[4], shA[4];
#pragma unroll
    for (int g = 0; g < 4; g++) {
        scA[g] = *reinterpret_cast<const float4 *>(a.s1 + wcA * 32 + 8 * g + 4 * lh);
        shA[g] = *reinterpret_cast<const float4 *>(a.h1 + wcA * 32 + 8 * g + 4 * lh);
    }
    // ... and of phase B (behind the loop of A these sixteen loads per lane queued up at the address unit in front of the
    // first weight stages of phase B)
    const int wpB = wave % WPB, wcB = wave / WPB;
    float4 scB[TCB][4], shB[TCB][4];
#pragma unroll
    for (int i = 0; i < TCB; i++)
#pragma unroll
        for (int g = 0; g < 4; g++) {
            scB[i][g] = *reinterpret_cast<const float4 *>(a.s2 + (wcB * TCB + i) * 32 + 8 * g + 4 * lh);
            shB[i][g] = *reinterpret_cast<const float4 *>(a.h2 + (wcB * TCB + i) * 32 + 8 * g + 4 * lh);
        }
#pragma unroll
    for (int s = 0; s < NSA - 1; s++) issueA(s, (unsigned)(s * XROWB), s < nA);

    // tap addresses of phase B (computed under the first DMAs): ax[j][t] = LDS byte address, plane 0, k-step 0, of tap t
    // of this lane's pixel in pixel block j, or of the zero row when that tap lies outside the image / the tile
    unsigned ax[TPB][9];
#pragma unroll
    for (int j = 0; j < TPB; j++) {
        const int mloc = (wpB * TPB + j) * 32 + lr, m = p0 + mloc;
        uint32_t t, wq, nn, hq;
        a.dw.divmod((uint32_t)m, t, wq);
        a.dh.divmod(t, nn, hq);
        const int h = (int)hq, w = (int)wq;
        const unsigned inside = m < pend ? 1u : 0u;
        const unsigned hok[3] = {inside & (h >= 1 ? 1u : 0u), inside, inside & (h + 1 < a.H ? 1u : 0u)};
        const unsigned wok[3] = {w >= 1 ? 1u : 0u, 1u, w + 1 < W ? 1u : 0u};
        const unsigned zero_base = lds_addr(t1) + PRA * 128;
#pragma unroll
        for (int tp = 0; tp < 9; tp++) {
            const int r = tp / 3, sx = tp % 3;
            const int row = mloc + r * W + sx;
            const unsigned real = lds_addr(t1) + (unsigned)row * 128u + (unsigned)((lh ^ swz<128>(row)) << 4);
            const unsigned zero_row = zero_base + (real & 255u);
            ax[j][tp] = zero_row + ((0u - (hok[r] & wok[sx])) & (real - zero_row));
        }
    }
    // the compiler's own bookkeeping learns here that the BN constants have arrived (they are older than every DMA above)
#pragma unroll
    for (int g = 0; g < 4; g++) asm volatile("" ::"v"(scA[g].x), "v"(scA[g].w), "v"(shA[g].x), "v"(shA[g].w));
#pragma unroll
    for (int i = 0; i < TCB; i++)
#pragma unroll
        for (int g = 0; g < 4; g++) asm volatile("" ::"v"(scB[i][g].x), "v"(scB[i][g].w), "v"(shB[i][g].x), "v"(shB[i][g].w));

    {
        f32x16_t acc[TPA];
#pragma unroll
        for (int j = 0; j < TPA; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[j][e] = 0.f;
        const unsigned fsw = (unsigned)swz<XROWB>(lr);
        const unsigned fx0 = lds_addr(ringA) + (unsigned)((wpA * TPA * 32 + lr) * XROWB) + ((lh ^ fsw) << 4);
        const unsigned fw0 = lds_addr(ringA) + (unsigned)(PRA * XROWB + (wcA * 32 + lr) * XROWB) + ((lh ^ fsw) << 4);
        u32x4_t fa[2], fb[2][TPA];
        auto readA = [&](auto SET, unsigned kx, unsigned sb) {
            constexpr int set = decltype(SET)::value;
            const unsigned aw = xor_add(fw0, kx, sb), axx = xor_add(fx0, kx, sb);
            lds_read16<0>(fa[set], aw);
            static_for<TPA>([&](auto J) { lds_read16<decltype(J)::value * 32 * XROWB>(fb[set][decltype(J)::value], axx); });
        };
        auto mmaA = [&](auto SET) {
            constexpr int set = decltype(SET)::value;
            landed(fa[set]);
            static_for<TPA>([&](auto J) { landed(fb[set][decltype(J)::value]); });
            static_for<TPA>([&](auto J) { Mma<bf16_t>::run(acc[decltype(J)::value], fa[set], fb[set][decltype(J)::value]); });
        };
        int slot = 0, islot = NSA - 1;
        for (int s = 0; s < nA; s++) {
            wait_vmcnt<(NSA - 2) * LA>();                 // this wave's share of stage s has landed
            __builtin_amdgcn_s_barrier();                 // ... everyone's; and nobody still reads stage s - 1, whose slot is refilled now
            issueA(islot, (unsigned)((s + NSA - 1) * XROWB), s + NSA - 1 < nA);
            const unsigned sb = (unsigned)(slot * SLOTA);
            readA(I0{}, 0u, sb);
            readA(I1{}, 32u, sb);
            wait_lgkmcnt<1 + TPA>();
            mmaA(I0{});
            wait_lgkmcnt<0>();
            mmaA(I1{});
            slot = slot + 1 == NSA ? 0 : slot + 1;
            islot = islot + 1 == NSA ? 0 : islot + 1;
        }
        wait_vmcnt<0>();
        __syncthreads();                                  // the ring is dead: its space becomes t1 and the ring of phase B
        // zero rows of the t1 planes (no DMA of phase B writes them) and first weight stages of phase B, all under the
        // epilogue of A
        if (tid < CH * 64) *reinterpret_cast<unsigned *>(t1 + (tid >> 6) * PLANE1 + PRA * 128 + (tid & 63) * 4) = 0u;
#pragma unroll
        for (int s = 0; s < NSB - 1; s++) issueB(s, s, s < nB);
        // ---- epilogue of A
#pragma unroll
        for (int j = 0; j < TPA; j++) {
            const int row = (wpA * TPA + j) * 32 + lr;
            if (row < PRA) {
#pragma unroll
                for (int g = 0; g < 4; g++) park(acc[j], g, scA[g], shA[g], PLANE1, row, wcA * 32 + 8 * g + 4 * lh);
            }
        }
        wait_lgkmcnt<0>();
    }
    __builtin_amdgcn_s_barrier();                         // t1 is complete (every wave's stores have been executed)

    // ================================================================ phase B: t2 = relu(bn2(conv3x3(t1)))
    // phase C state that is set up before the epilogue of B
    const int wpC = wave % WPC, wcC = wave / WPC;
    const int mwC = p0 + wpC * TPC * 32;
    const bf16_t *__restrict__ xres = static_cast<const bf16_t *>(a.x);
    ResidualRegs<bf16_t, TPC, 1> res[2];                  // shortcut rows of the current and of the next pass
    res[0].on = res[1].on = true;
    constexpr int NRES = TPC * 2;                         // loads per lane and pass, always issued (clamped addresses)
    auto load_res = [&](auto SET, int q) {
        constexpr int set = decltype(SET)::value;
        const int erow = lane >> 2, cb = min(q * PC + wcC * 32, C4 - 32) + (lane & 3) * 8;     // beyond the last pass: any valid channels
#pragma unroll
        for (int j = 0; j < TPC; j++)
#pragma unroll
            for (int ps = 0; ps < 2; ps++) {
                const int m = min(mwC + j * 32 + erow + ps * 16, pend - 1);                      // rows beyond the tile are never stored
                res[set].r[j][ps].load(xres + (size_t)m * C4 + cb);
            }
    };
    {
        f32x16_t acc[TCB][TPB];
#pragma unroll
        for (int i = 0; i < TCB; i++)
#pragma unroll
            for (int j = 0; j < TPB; j++)
#pragma unroll
                for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;
        const unsigned fw0 = lds_addr(ring) + (unsigned)((wcB * TCB * 32 + lr) * 128) + ((lh ^ (unsigned)swz<128>(lr)) << 4);
        u32x4_t fa[2][TCB], fb[2][TPB];
        auto readB = [&](auto SET, auto TAP, unsigned kx, unsigned sb, unsigned pb) {
            constexpr int set = decltype(SET)::value, tp = decltype(TAP)::value;
            const unsigned aw = xor_add(fw0, kx, sb);
            static_for<TCB>([&](auto I) { lds_read16<decltype(I)::value * 32 * 128>(fa[set][decltype(I)::value], aw); });
            static_for<TPB>([&](auto J) { lds_read16<0>(fb[set][decltype(J)::value], xor_add(ax[decltype(J)::value][tp], kx, pb)); });
        };
        auto mmaB = [&](auto SET) {
            constexpr int set = decltype(SET)::value;
            static_for<TCB>([&](auto I) { landed(fa[set][decltype(I)::value]); });
            static_for<TPB>([&](auto J) { landed(fb[set][decltype(J)::value]); });
            static_for<TCB * TPB>([&](auto Q) {
                constexpr int q = decltype(Q)::value, i = q / TPB, j = q % TPB;
                Mma<bf16_t>::run(acc[i][j], fa[set][i], fb[set][j]);
            });
        };
        int slot = 0, islot = NSB - 1, sidx = 0;
        for (int c = 0; c < CH; c++) {
            const unsigned pb = (unsigned)(c * PLANE1);
            static_for<9>([&](auto TAP) {
                wait_vmcnt<(NSB - 2) * LB>();
                __builtin_amdgcn_s_barrier();
                issueB(islot, sidx + NSB - 1, sidx + NSB - 1 < nB);
                const unsigned sb = (unsigned)(slot * SLOTB);
                readB(I0{}, TAP, 0u, sb, pb);
                readB(I1{}, TAP, 32u, sb, pb);
                wait_lgkmcnt<TCB + TPB>();
                mmaB(I0{});
                readB(I0{}, TAP, 64u, sb, pb);
                wait_lgkmcnt<TCB + TPB>();
                mmaB(I1{});
                readB(I1{}, TAP, 96u, sb, pb);
                wait_lgkmcnt<TCB + TPB>();
                mmaB(I0{});
                wait_lgkmcnt<0>();
                mmaB(I1{});
                slot = slot + 1 == NSB ? 0 : slot + 1;
                islot = islot + 1 == NSB ? 0 : islot + 1;
                sidx++;
            });
        }
        wait_vmcnt<0>();
        __syncthreads();                                  // every wave is done with t1 and the ring: t2 goes over t1
        // first W3 rows and shortcut rows of phase C, under the epilogue of B
        issueC(0, 0, true);
        load_res(I0{}, 0);
        // ---- epilogue of B: into the t2 planes (same row layout, NBO * 32 rows per plane)
#pragma unroll
        for (int i = 0; i < TCB; i++)
#pragma unroll
            for (int j = 0; j < TPB; j++) {
                const int row = (wpB * TPB + j) * 32 + lr;
#pragma unroll
                for (int g = 0; g < 4; g++) park(acc[i][j], g, scB[i][g], shB[i][g], PLANE2, row, (wcB * TCB + i) * 32 + 8 * g + 4 * lh);
            }
        wait_lgkmcnt<0>();
    }

    // ================================================================ phase C: y = relu(bn3(t2 . W3) + x), PC channels per pass
    // The W3 rows of a pass (PC x WM, 16 KB) sit in one of two buffers; the next pass's rows and shortcut rows are
    // fetched while the current pass is contracted.  Right before its epilogue a wave waits until only the shortcut
    // loads of the NEXT pass may be outstanding: its share of the next W3 rows and its own shortcut rows are then
    // here, and the barrier behind the epilogue publishes the W3 rows.  No wait ever has to count the epilogue's stores.
    float *const strips = reinterpret_cast<float *>(ringC + 2 * PCBUF);
    ConvArgs ca;                                          // what the shared epilogue reads
    ca.y = a.y; ca.res = a.x; ca.scale = a.s3; ca.shift = a.h3; ca.prepool = nullptr; ca.argmax = nullptr;
    ca.Cout = C4; ca.ldy = C4; ca.P = pend; ca.act = SOL_ACT_RELU; ca.pool = 0;
    wait_vmcnt<NRES>();                                   // the first W3 rows (this wave's share) are here
    __builtin_amdgcn_s_barrier();                         // ... everyone's, and t2 is complete
    {
        f32x16_t acc[1][TPC];
        const unsigned fw0 = lds_addr(ringC) + (unsigned)((wcC * 32 + lr) * 128) + ((lh ^ (unsigned)swz<128>(lr)) << 4);
        const unsigned fx0 = lds_addr(t1) + (unsigned)((wpC * TPC * 32 + lr) * 128) + ((lh ^ (unsigned)swz<128>(lr)) << 4);
        u32x4_t fa[2], fb[2][TPC];
        auto readC = [&](auto SET, unsigned kx, unsigned sb, unsigned pb) {
            constexpr int set = decltype(SET)::value;
            const unsigned aw = xor_add(fw0, kx, sb), axx = xor_add(fx0, kx, pb);
            lds_read16<0>(fa[set], aw);
            static_for<TPC>([&](auto J) { lds_read16<decltype(J)::value * 32 * 128>(fb[set][decltype(J)::value], axx); });
        };
        auto mmaC = [&](auto SET) {
            constexpr int set = decltype(SET)::value;
            landed(fa[set]);
            static_for<TPC>([&](auto J) { landed(fb[set][decltype(J)::value]); });
            static_for<TPC>([&](auto J) { Mma<bf16_t>::run(acc[0][decltype(J)::value], fa[set], fb[set][decltype(J)::value]); });
        };
        for (int q0 = 0; q0 < npass; q0 += 2) {
            static_for<2>([&](auto PARITY) {
                constexpr int par = decltype(PARITY)::value;
                const int q = q0 + par;
                if (q < npass) {
                    const int cw = q * PC + wcC * 32;
                    issueC(par ^ 1, q + 1, q + 1 < npass);
                    load_res(std::integral_constant<int, par ^ 1>{}, q + 1);
#pragma unroll
                    for (int j = 0; j < TPC; j++)
#pragma unroll
                        for (int e = 0; e < 16; e++) acc[0][j][e] = 0.f;
                    const unsigned bufo = (unsigned)(par * PCBUF);
                    static_for<CH>([&](auto CI) {
                        constexpr int c = decltype(CI)::value;
                        const unsigned sb = bufo + (unsigned)(c * PC * 128), pb = (unsigned)(c * PLANE2);
                        readC(I0{}, 0u, sb, pb);
                        readC(I1{}, 32u, sb, pb);
                        wait_lgkmcnt<1 + TPC>();
                        mmaC(I0{});
                        readC(I0{}, 64u, sb, pb);
                        wait_lgkmcnt<1 + TPC>();
                        mmaC(I1{});
                        readC(I1{}, 96u, sb, pb);
                        wait_lgkmcnt<1 + TPC>();
                        mmaC(I0{});
                        wait_lgkmcnt<0>();
                        mmaC(I1{});
                    });
                    wait_vmcnt<NRES>();                   // all but the next pass's shortcut loads: the next W3 rows, this pass's shortcut rows
                    const Affine8 aff = load_affine_unconditional<1>(ca, lane, cw);
                    conv_epilogue_auto<bf16_t, TPC, 1>(ca, acc, strips, wave, lane, mwC, cw, aff, LinearRows{pend}, res[par]);
                    __builtin_amdgcn_s_barrier();         // everyone's share has landed; everyone is done with this pass's buffer
                }
            });
        }
    }
    wait_vmcnt<0>();
#endif
}

// One configuration per mid width: 64 channels (56-wide images: up to 63 columns), 128 channels (up to 31 columns)
template <int WM> struct BlockCfg;
template <> struct BlockCfg<64> { static constexpr int PRA = 384, NBO = 8; };
template <> struct BlockCfg<128> { static constexpr int PRA = 288, NBO = 8; };

static int block_tile_pixels(int WM, int W) {
    const int pra = WM == 64 ? BlockCfg<64>::PRA : BlockCfg<128>::PRA;
    return std::min(256, pra - 2 * W - 2);
}

// bf16; mid width 64 or 128; C4 a multiple of 128; stride 1; tensors below 2 GB (32-bit byte offsets)
bool block_kernel_applies(int dt, int N, int H, int W, int C4, int WM) {
    if (dt != SOL_BF16 || !(WM == 64 || WM == 128) || C4 % 128 != 0 || C4 < 128) return false;
    if ((double)N * H * W * C4 * 2.0 >= 2147483648.0) return false;
    return block_tile_pixels(WM, W) >= 64;
}

sol_status launch_conv_block(const BlockLaunch &b, hipStream_t st) {
    SOL_REQUIRE(block_kernel_applies(SOL_BF16, b.N, b.H, b.W, b.C4, b.WM), SOL_ERR_UNSUPPORTED, "fused bottleneck: unsupported shape");
    BlockArgs a;
    a.x = b.x; a.y = b.y; a.w1 = b.w1; a.w2 = b.w2; a.w3 = b.w3;
    a.s1 = b.s1; a.h1 = b.h1; a.s2 = b.s2; a.h2 = b.h2; a.s3 = b.s3; a.h3 = b.h3;
    a.P = b.N * b.H * b.W; a.H = b.H; a.W = b.W; a.C4 = b.C4;
    if (a.P <= 0) return SOL_OK;
    a.bp = block_tile_pixels(b.WM, b.W);
    a.ntiles = ceil_div(a.P, a.bp);
    a.dw = FastDiv((uint32_t)b.W);
    a.dh = FastDiv((uint32_t)b.H);
    const int grid = ((a.ntiles + 7) / 8) * 8;
    //                                     NW  WM  PRA  NBO WPA TPA WPB TPB TCB NSA NSB
    if (b.WM == 64)
        hipLaunchKernelGGL((conv_block_kernel<8, 64, 384, 8, 4, 3, 4, 2, 1, 5, 4>), dim3(grid), dim3(512), 0, st, a);
    else
        hipLaunchKernelGGL((conv_block_kernel<8, 128, 288, 8, 2, 5, 4, 2, 2, 5, 4>), dim3(grid), dim3(512), 0, st, a);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

}  // namespace sol

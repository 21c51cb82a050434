// Expand -> reduce pair across two consecutive bottlenecks as ONE depth-first kernel (gfx950, bf16):
//
//     y = relu(s3 * (t . W3) + h3 + r)        [P][C4]     1x1, WM -> C4 channels, + shortcut r   (last layer of block i)
//     z = relu(s1 * (y . W1) + h1)            [P][WZ]     1x1, C4 -> WZ channels                 (first layer of block i+1)
//
// Run as two layers, y -- the widest tensor of the stage -- is written, read back by a second launch, and both launches
// pay their ramp-up and tail; their reductions are short (WM) and long (C4), and the second one leaves a quarter of the
// CUs idle in the 14x14 stage.  Here a workgroup owns 64 pixels and ALL channels: y is produced in passes of 128 channels,
// stored (the next shortcut still needs it), and each pass is contracted into the z accumulators right away while it
// sits in LDS as bf16 -- the paper's depth-first processing (Sec. III-A: a chain of layers is run over a block of data
// while it is in registers and on-chip memory), with the rounding point of the stored tensor kept.
//
// One pipeline for everything: operands reach LDS by DMA (buffer_load ... lds) into a ring of 16 KB slots, one
// workgroup barrier per two slots, fragment reads as opaque statements ordered by hand, every DMA issued unconditionally
// (beyond the end through a size-0 resource) so that the in-order vmcnt bookkeeping is static.  A pass is eight slots
// (two per barrier) for WZ = 256:
//   Y-stage k (k < 4):   W3[pass rows 0..127][64 k .. 64 k + 63]      128 rows x 128 B;  y-pass += t[:, plane k] . that
//   Z-stage u (u < 4):   W1[rows 0..255][128 pass + 32 u .. + 31]     256 rows x  64 B;  z += y-pass[:, 32 u ..] . that
// and twelve for WZ = 512: the W1 rows of a 32-channel group are then two adjacent slots (rows 0..255, 256..511).
// Between them the pass's accumulators get affine + shortcut + ReLU, are rounded and parked in LDS (the shortcut rows
// and the affine constants also come from LDS: the rows by DMA one pass ahead, the constants once); the store of the
// pass to y is issued from LDS behind the MFMAs of the first Z-stage.  A wave keeps its pixels of t as fragments in registers.
#include <algorithm>

#include "conv_common.h"

namespace sol {

struct XrArgs {
    const void *t, *r;                 // input of the expand layer [P][WM]; its shortcut [P][C4]
    void *y, *z;                       // [P][C4], [P][WZ]
    const void *w3, *w1;               // packed [C4][WM], [WZ][C4]
    const float *s3, *h3, *s1, *h1;    // folded BN + bias (scale, shift) of the two layers
    int P, C4, ntiles;
};

__device__ __forceinline__ void lds_read8(unsigned long long &dst, unsigned addr) {
    asm volatile("ds_read_b64 %0, %1" : "=&v"(dst) : "v"(addr));
}

template <int WM, int WZ, int NS>
__global__ void __launch_bounds__(512) conv_xr_kernel(const XrArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)
    using namespace lds_pipe;
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    constexpr int NW = 8, BP = 64, PC = 128;
    constexpr int ZH = WZ / 256;                                      // 256-row halves of a 32-channel group of W1 rows
    constexpr int UY = WM / 64, UZ = PC / 32 * ZH, UPP = UY + UZ;     // slots of a pass
    constexpr int SP = UPP / 2;                                       // stages (two slots, one barrier) of a pass
    constexpr int NB = WZ / 128;                                      // 32-channel blocks of z per wave
    constexpr int SLOT = 16384, L = SLOT / 1024 / NW;                 // DMA instructions per wave and slot
    constexpr int PLANE = BP * 128;                                   // 64 pixels x 64 channels
    // LDS: the parked y pass, the shortcut rows of a pass, the affine constants of y, the ring.  The pixel tile t is needed
    // in LDS only until every wave has taken its fragments into registers (it is re-read by every pass: 64 registers save
    // half of the LDS traffic of the Y-stages); it lands in the last two ring slots, which join the ring afterwards.
    constexpr int YCH_OFF = 0, RB_OFF = YCH_OFF + 2 * PLANE, CST_OFF = RB_OFF + 2 * PLANE, RING_OFF = CST_OFF + 8192,
                  T_OFF = RING_OFF + (NS - 2) * SLOT, LDSB = RING_OFF + NS * SLOT + 1024;
    static_assert(WM == 256 && (WZ == 256 || WZ == 512), "slots of 16 KB: 128 rows of W3 x 128 B, 256 rows of W1 x 64 B");
    static_assert(NS == 6 && LDSB <= 160 * 1024 && UY * PLANE == 2 * SLOT, "ring: three stages of two slots");
    static_assert(NW * 32 * (64 + 4) * 4 <= NS * SLOT, "the epilogue strips of z go over the dead ring");

    __shared__ __align__(1024) unsigned char lds[LDSB];
    unsigned char *const ring = lds + RING_OFF, *const dump = lds + RING_OFF + NS * SLOT;

    asm volatile("" ::"s"(a.t), "s"(a.r), "s"(a.y), "s"(a.z), "s"(a.w3), "s"(a.w1), "s"(a.s3), "s"(a.h3), "s"(a.s1), "s"(a.h1),
                 "s"(a.P), "s"(a.C4), "s"(a.ntiles));

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lr = lane & 31, lh = lane >> 5;
    const int wp = wave & 1, wc = wave >> 1;                          // pixel block (of 2) and channel group (of 4) of this wave
    const int tile = (int)(blockIdx.x & 7) * ((a.ntiles + 7) >> 3) + (int)(blockIdx.x >> 3);   // a contiguous run of tiles per XCD
    if (tile >= a.ntiles) return;
    const int C4 = a.C4, p0 = tile * BP;
    const int npass = C4 / PC;
    // The workgroups of an XCD all stream the same weights; started on the same pass they ask its L2 for the same lines
    // at the same time.  Each tile therefore walks the passes in its own rotation (pass rot first): y passes are
    // independent, and z adds them in an order that is fixed per tile.
    const int rot = tile % npass;
    auto pe = [&](int q) { const int e = q + rot; return e >= npass ? e - npass : e; };   // q-th pass of this tile's walk (q <= npass)

    const __amdgpu_buffer_rsrc_t tr = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.t), 0, a.P * WM * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t rr = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.r), 0, a.P * C4 * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t w3r = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.w3), 0, C4 * WM * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t w1r = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.w1), 0, WZ * C4 * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t s3r = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.s3), 0, C4 * 4, 0x00020000);
    const __amdgpu_buffer_rsrc_t h3r = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.h3), 0, C4 * 4, 0x00020000);
    const __amdgpu_buffer_rsrc_t nullr = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.t), 0, 0, 0x00020000);   // size 0: zeros

    // both weight sets are cold when the launch starts: one dword per 128-byte line, spread over the XCD's workgroups
    warm_l2(static_cast<const unsigned char *>(a.w3), (unsigned)(C4 * WM * 2), dump + (wave & 3) * 256, tid, NW * 64);
    warm_l2(static_cast<const unsigned char *>(a.w1), (unsigned)(WZ * C4 * 2), dump + (wave & 3) * 256, tid, NW * 64);

    // ---- DMA lane offsets.  Rows of 128 bytes: one instruction = 8 rows x 8 slots of 16 bytes; rows of 64 bytes: 16 rows x 4.
    const int ls8 = lane & 7, lrow8 = lane >> 3, ls4 = lane & 3, lrow16 = lane >> 2;
    unsigned woY[L], woZ[L], roR[L], toT[UY];
#pragma unroll
    for (int i = 0; i < L; i++) {
        const int idx = wave * L + i;
        const int rowy = idx * 8 + lrow8;                             // W3 row of the pass
        woY[i] = (unsigned)rowy * (unsigned)(WM * 2) + (unsigned)((ls8 ^ swz<128>(rowy)) << 4);
        const int rowz = idx * 16 + lrow16;                           // W1 row
        woZ[i] = (unsigned)rowz * (unsigned)(C4 * 2) + (unsigned)((ls4 ^ swz<64>(rowz)) << 4);
        const int rowr = (idx & 7) * 8 + lrow8;                       // shortcut: plane idx / 8 of the pass, pixel rowr
        roR[i] = p0 + rowr < a.P ? (unsigned)(p0 + rowr) * (unsigned)(C4 * 2) + (unsigned)((idx >> 3) * 128) + (unsigned)((ls8 ^ swz<128>(rowr)) << 4)
                                 : 0xffffffffu;   // pixels beyond the tensor (ragged last tile): the range check returns zeros
    }
#pragma unroll
    for (int i = 0; i < UY; i++) {
        const int idx = wave * UY + i, row = (idx & 7) * 8 + lrow8;   // t: plane idx / 8, pixel row
        toT[i] = p0 + row < a.P ? (unsigned)(p0 + row) * (unsigned)(WM * 2) + (unsigned)((idx >> 3) * 128) + (unsigned)((ls8 ^ swz<128>(row)) << 4) : 0xffffffffu;
    }
    // I-th DMA instruction of this wave for slot POS of pass q: W3 rows (POS < UY) or W1 rows
    auto issue_one = [&](auto POS, auto I, int slot, int q, bool real) {
        constexpr int pos = decltype(POS)::value, i = decltype(I)::value;
        unsigned char *dst = ring + slot * SLOT + (wave * L + i) * 1024;
        if constexpr (pos < UY) {
            const unsigned soff = (unsigned)(pe(q) * PC) * (unsigned)(WM * 2) + (unsigned)(pos * 128);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(real ? w3r : nullr, (__attribute__((address_space(3))) void *)dst, 16, woY[i], soff, 0, 0);
        } else {
            constexpr int zi = pos - UY, u = zi / ZH, h = zi % ZH;   // 32-channel group of the pass, half of the W1 rows
            const unsigned soff = (unsigned)((pe(q) * PC + u * 32) * 2) + (unsigned)h * (unsigned)(256 * 2) * (unsigned)C4;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(real ? w1r : nullr, (__attribute__((address_space(3))) void *)dst, 16, woZ[i], soff, 0, 0);
        }
    };
    auto issue_unit = [&](auto POS, int slot, int q, bool real) {
        static_for<L>([&](auto I) { issue_one(POS, I, slot, q, real); });
    };
    auto issue_shortcut = [&](int q, bool real) {
        static_for<L>([&](auto I) {
            constexpr int i = decltype(I)::value;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(real ? rr : nullr, (__attribute__((address_space(3))) void *)(lds + RB_OFF + (wave * L + i) * 1024), 16,
                                                     roR[i], (unsigned)(pe(q) * PC * 2), 0, 0);
        });
    };

    // ---- prologue: the pixel tile, the affine constants of y, the first shortcut rows, the first NS - 1 slots
    static_for<UY>([&](auto I) {
        constexpr int i = decltype(I)::value;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(tr, (__attribute__((address_space(3))) void *)(lds + T_OFF + (wave * UY + i) * 1024), 16, toT[i], 0u, 0, 0);
    });
    // waves 0-3: 1 KB each of s3 (channels 256 w ..), waves 4-7: of h3; beyond C4 the resource returns zeros
    __builtin_amdgcn_raw_ptr_buffer_load_lds(wave < 4 ? s3r : h3r, (__attribute__((address_space(3))) void *)(lds + CST_OFF + wave * 1024), 16,
                                             (unsigned)((wave & 3) * 1024 + lane * 16), 0u, 0, 0);
    issue_shortcut(0, true);
    static_for<NS - 2>([&](auto S) {
        constexpr int s = decltype(S)::value;
        issue_unit(std::integral_constant<int, s % UPP>{}, s, s / UPP, s / UPP < npass);
    });

    // fragment addresses (k-step / slot / plane are added at the point of use)
    const unsigned sw128 = (unsigned)swz<128>(lr), sw64 = (unsigned)swz<64>(lr);
    const unsigned fwy0 = lds_addr(ring) + (unsigned)((wc * 32 + lr) * 128) + ((lh ^ sw128) << 4);       // W3 rows of this wave's 32 channels
    const unsigned fwz0 = lds_addr(ring) + (unsigned)((wc * (WZ / 4) + lr) * 64) + ((lh ^ sw64) << 4);   // W1 rows of its WZ / 4 channels of z
    const unsigned fpx0 = (unsigned)((wp * 32 + lr) * 128) + ((lh ^ sw128) << 4);                        // its pixel rows inside a plane
    const unsigned ft0 = lds_addr(lds + T_OFF) + fpx0, fy0 = lds_addr(lds + YCH_OFF) + fpx0;
    // epilogue of a y pass: this lane's pixel row, channel group g -> 4 channels 8 g + 4 lh of the wave's 32
    const int erow = wp * 32 + lr;
    unsigned eoff[4];                                                  // byte offset inside the two planes of a pass
#pragma unroll
    for (int g = 0; g < 4; g++) {
        const int ch = wc * 32 + 8 * g + 4 * lh;
        eoff[g] = (unsigned)((ch >> 6) * PLANE + erow * 128) + (unsigned)((((ch & 63) >> 3) ^ swz<128>(erow)) << 4) + (unsigned)((ch & 7) * 2);
    }
    // store of a y pass from LDS: 16 bytes of plane 0 and of plane 1 per lane
    // (a lane whose pixel lies beyond the tensor -- ragged last tile -- repeats the store of the last pixel, same bytes to the
    // same place: every wave issues its two stores, as the static counts assume)
    const int srow = min(tid >> 3, a.P - 1 - p0), sls = tid & 7;
    const unsigned ysrc = lds_addr(lds + YCH_OFF) + (unsigned)(srow * 128) + (unsigned)((sls ^ swz<128>(srow)) << 4);
    unsigned char *const ydst = static_cast<unsigned char *>(a.y) + ((size_t)(p0 + srow) * C4 + sls * 8) * 2;

    // ---- this wave's 32 pixels of t, all 256 channels, as MFMA fragments: [plane][k-step]
    u32x4_t ft[UY][4];
    wait_vmcnt<1 + L + (NS - 2) * L>();                               // the tile has landed (this wave's share) ...
    __builtin_amdgcn_s_barrier();                                      // ... everyone's
    static_for<UY>([&](auto C) {
        static_for<4>([&](auto K) {
            constexpr int c = decltype(C)::value, k = decltype(K)::value;
            lds_read16<c * PLANE>(ft[c][k], (ft0 ^ (unsigned)(k * 32)));
        });
    });
    wait_lgkmcnt<0>();
    static_for<UY>([&](auto C) { static_for<4>([&](auto K) { landed(ft[decltype(C)::value][decltype(K)::value]); }); });
    __builtin_amdgcn_s_barrier();                                      // every wave has its fragments: the tile's space joins the ring

    f32x16_t zacc[NB / 2][2][1], yacc[2];   // z: block b of the wave = zacc[b / 2][b % 2]; y: two accumulators taking alternate k-steps (a wave's MFMAs of a Y-stage would otherwise form one dependent chain)
#pragma unroll
    for (int b = 0; b < NB; b++)
#pragma unroll
        for (int e = 0; e < 16; e++) zacc[b / 2][b % 2][0][e] = 0.f;

    // A wave has one (Y) or two (Z) MFMAs per k-step: too little to hide an LDS round trip behind.  All fragments of a
    // stage (two slots) are therefore requested at once and the MFMAs follow back to back, each waiting only for its own.
    u32x4_t fw[8], fz[4][2], fyy[4];
    auto stageY = [&](auto C0, unsigned sb, auto &&between) {          // slots of planes C0 and C0 + 1; between(j) after MFMA pair j
        constexpr int c0 = decltype(C0)::value;
        static_for<8>([&](auto K) {
            constexpr int k = decltype(K)::value;
            lds_read16<(k >> 2) * SLOT>(fw[k], xor_add(fwy0, (unsigned)((k & 3) * 32), sb));
        });
        static_for<8>([&](auto K) {
            constexpr int k = decltype(K)::value;
            wait_lgkmcnt<7 - k>();
            landed(fw[k]);
            Mma<bf16_t>::run(yacc[k & 1], fw[k], ft[c0 + (k >> 2)][k & 3]);
            if constexpr (k & 1) between(std::integral_constant<int, k / 2>{});
        });
    };
    auto stageZ = [&](auto U0, unsigned sb, auto &&between) {          // slots of the 32-channel groups U0 and U0 + 1 of the pass
        constexpr int u0 = decltype(U0)::value;
        static_assert(u0 % 2 == 0, "both groups lie in one plane of the parked pass");
        constexpr unsigned pb = (unsigned)((u0 >> 1) * PLANE);
        static_for<4>([&](auto K) {
            constexpr int k = decltype(K)::value;                      // k-step k & 1 of slot k >> 1
            const unsigned aw = xor_add(fwz0, (unsigned)((k & 1) * 32), sb);
            lds_read16<(k >> 1) * SLOT>(fz[k][0], aw);
            lds_read16<(k >> 1) * SLOT + 32 * 64>(fz[k][1], aw);
            lds_read16<0>(fyy[k], xor_add(fy0, (unsigned)(k * 32), pb));
        });
        static_for<4>([&](auto K) {
            constexpr int k = decltype(K)::value;
            wait_lgkmcnt<9 - 3 * k>();
            landed(fz[k][0]);
            landed(fz[k][1]);
            landed(fyy[k]);
            Mma<bf16_t>::run(zacc[0][0][0], fz[k][0], fyy[k]);
            Mma<bf16_t>::run(zacc[0][1][0], fz[k][1], fyy[k]);
            between(K);
        });
    };
    // WZ = 512: a stage is ONE 32-channel group of the pass, all 512 rows of W1 (two adjacent slots): two k-steps, four blocks
    auto stageZ2 = [&](auto U, unsigned sb, auto &&between) {
        constexpr int u = decltype(U)::value;
        constexpr unsigned pb = (unsigned)((u >> 1) * PLANE);
        u32x4_t gz[2][4];
        static_for<2>([&](auto K) {
            constexpr int k = decltype(K)::value;
            const unsigned aw = xor_add(fwz0, (unsigned)(k * 32), sb);
            static_for<4>([&](auto B) { lds_read16<decltype(B)::value * 32 * 64>(gz[k][decltype(B)::value], aw); });
            lds_read16<0>(fyy[k], xor_add(fy0, (unsigned)(((u & 1) * 2 + k) * 32), pb));
        });
        static_for<2>([&](auto K) {
            constexpr int k = decltype(K)::value;
            wait_lgkmcnt<5 - 5 * k>();
            static_for<4>([&](auto B) { landed(gz[k][decltype(B)::value]); });
            landed(fyy[k]);
            static_for<4>([&](auto B) {
                constexpr int b = decltype(B)::value;
                Mma<bf16_t>::run(zacc[b / 2][b % 2][0], gz[k][b], fyy[k]);
                if constexpr (b & 1) between(std::integral_constant<int, 2 * k + b / 2>{});
            });
        });
    };

    // A stage = two slots = one barrier (with one slot per barrier the waits, the barrier and the DMA issue cost as much as
    // the four MFMAs of a slot).  A pass is SP stages: Y 0-1, Y 2-3 + the epilogue of y, then the Z stages (two for
    // WZ = 256: groups 0-1, 2-3; four for WZ = 512: one group each), the first of them behind the store of the pass and the
    // fetch of the next shortcut rows.  Stage s issues the slots of stage s + 2.
    int slot = 0, islot = NS - 2;
    for (int q = 0; q < npass; q++) {
        static_for<SP>([&](auto POS) {
            constexpr int pos = decltype(POS)::value;
            // in flight behind this stage's slots: the two slots issued one stage ago, and what the first Z stage issues at
            // its END (the two stores of the y pass and the next shortcut rows), which is behind that stage's own slots and
            // in front of the next stage's: it counts for the two stages that follow a first Z stage
            constexpr int N0 = 2 * L, N = N0 + ((pos == 3 || pos == 4 % SP) ? 2 + L : 0);
            if constexpr (pos == 0) {                                  // no first Z stage in front of the first pass
                if (q == 0) wait_vmcnt<N0>(); else wait_vmcnt<N>();
            } else {
                wait_vmcnt<N>();                                       // this wave's share of both slots has landed
            }
            __builtin_amdgcn_s_barrier();                              // ... everyone's; and nobody still reads the slots refilled now
            // the four DMA instructions of the stage two ahead go out between this stage's MFMAs, one per MFMA pair: a wave
            // issues in order, and a DMA instruction waits its turn at the CU's address unit (about 18 cycles per KB, all
            // eight waves queue there right behind the barrier) -- time in which the matrix pipe would otherwise idle
            auto dma = [&](auto J) {
                constexpr int j = decltype(J)::value, ipos = ((pos + 2) % SP) * 2 + j / L, carry = (pos + 2) / SP;
                issue_one(std::integral_constant<int, ipos>{}, std::integral_constant<int, j % L>{}, islot + j / L, q + carry, q + carry < npass);
            };
            const unsigned sb = (unsigned)(slot * SLOT);
            if constexpr (pos < 2) {
                if constexpr (pos == 0) {
#pragma unroll
                    for (int e = 0; e < 16; e++) { yacc[0][e] = 0.f; yacc[1][e] = 0.f; }
                }
                stageY(std::integral_constant<int, 2 * pos>{}, sb, dma);
                if constexpr (pos == 1) {
                    // ---- the pass is contracted: affine + shortcut + ReLU, rounded, parked as the operand of the Z-stages
                    // (constants, shortcut rows: in LDS since the barrier above at the latest)
                    u32x4_t sc[4], sh[4];
                    unsigned long long rv[4];
                    const unsigned cst = lds_addr(lds + CST_OFF) + (unsigned)((pe(q) * PC + wc * 32 + 4 * lh) * 4);
                    const unsigned ych_base = lds_addr(lds + YCH_OFF), rb_base = lds_addr(lds + RB_OFF);
                    static_for<4>([&](auto G) {
                        constexpr int g = decltype(G)::value;
                        lds_read16<g * 32>(sc[g], cst);
                        lds_read16<4096 + g * 32>(sh[g], cst);
                        lds_read8(rv[g], rb_base + eoff[g]);
                    });
                    wait_lgkmcnt<0>();
                    static_for<4>([&](auto G) {
                        constexpr int g = decltype(G)::value;
                        landed(sc[g]);
                        landed(sh[g]);
                        asm volatile("" : "+v"(rv[g]));
                        const unsigned lo = (unsigned)rv[g], hi = (unsigned)(rv[g] >> 32);
                        float v0 = (yacc[0][4 * g] + yacc[1][4 * g]) * __uint_as_float(sc[g].x) + __uint_as_float(sh[g].x) + __uint_as_float(lo << 16);
                        float v1 = (yacc[0][4 * g + 1] + yacc[1][4 * g + 1]) * __uint_as_float(sc[g].y) + __uint_as_float(sh[g].y) + __uint_as_float(lo & 0xffff0000u);
                        float v2 = (yacc[0][4 * g + 2] + yacc[1][4 * g + 2]) * __uint_as_float(sc[g].z) + __uint_as_float(sh[g].z) + __uint_as_float(hi << 16);
                        float v3 = (yacc[0][4 * g + 3] + yacc[1][4 * g + 3]) * __uint_as_float(sc[g].w) + __uint_as_float(sh[g].w) + __uint_as_float(hi & 0xffff0000u);
                        v0 = __builtin_fmaxf(v0, 0.f); v1 = __builtin_fmaxf(v1, 0.f); v2 = __builtin_fmaxf(v2, 0.f); v3 = __builtin_fmaxf(v3, 0.f);   // one v_max each; a NaN becomes 0
                        const unsigned long long pk = (unsigned long long)pack_bf16x2(v0, v1) | ((unsigned long long)pack_bf16x2(v2, v3) << 32);
                        const unsigned ydst_lds = ych_base + eoff[g];
                        asm volatile("ds_write_b64 %0, %1" ::"v"(ydst_lds), "v"(pk) : "memory");
                    });
                    wait_lgkmcnt<0>();
                }
            } else {
                if constexpr (WZ == 256) stageZ(std::integral_constant<int, 2 * (pos - 2)>{}, sb, dma);
                else stageZ2(std::integral_constant<int, pos - 2>{}, sb, dma);
                if constexpr (pos == 2) {
                    // under this stage's MFMAs: the parked y pass goes to memory (two 16-byte pieces per lane, from LDS), and
                    // the next shortcut rows are fetched (every wave is past the epilogue that read the current ones)
                    u32x4_t v0, v1;
                    lds_read16<0>(v0, ysrc);
                    lds_read16<PLANE>(v1, ysrc);
                    wait_lgkmcnt<0>();
                    landed(v0);
                    landed(v1);
                    // opaque stores with a memory clobber: they keep their place among the DMAs, as the static counts assume
                    unsigned char *const yq = ydst + (size_t)pe(q) * (PC * 2);
                    asm volatile("global_store_dwordx4 %0, %1, off\n\tglobal_store_dwordx4 %0, %2, off offset:128" ::"v"(yq), "v"(v0), "v"(v1) : "memory");
                    issue_shortcut(q + 1, q + 1 < npass);
                }
            }
            slot = slot + 2 == NS ? 0 : slot + 2;
            islot = islot + 2 == NS ? 0 : islot + 2;
        });
    }
    // ---- z: through the shared epilogue (strips over the dead ring)
    ConvArgs ca;
    ca.y = a.z; ca.res = nullptr; ca.scale = a.s1; ca.shift = a.h1; ca.prepool = nullptr; ca.argmax = nullptr;
    ca.Cout = WZ; ca.ldy = WZ; ca.P = a.P; ca.act = SOL_ACT_RELU; ca.pool = 0;
    const int mw = p0 + wp * 32;
    ResidualRegs<bf16_t, 1, 2> none;
    none.on = false;
    wait_vmcnt<0>();
    wait_lgkmcnt<0>();
    __builtin_amdgcn_s_barrier();                                      // every wave is done with the ring
    static_for<NB / 2>([&](auto H) {                                   // 64 channels at a time through this wave's strip
        constexpr int h = decltype(H)::value;
        const int cw = wc * (WZ / 4) + h * 64;
        const Affine8 aff = load_affine_unconditional<2>(ca, lane, cw);
        conv_epilogue_auto<bf16_t, 1, 2>(ca, zacc[h], reinterpret_cast<float *>(ring), wave, lane, mw, cw, aff, LinearRows{a.P}, none);
    });
#endif
}

// bf16; 256 -> C4 -> 256 or 512 channels, C4 a multiple of 128 up to 1024 (the affine constants of y sit in 8 KB of LDS);
// any pixel count (tiles of 64, the last one ragged); tensors below 2 GB (32-bit byte offsets)
bool xr_kernel_applies(int dt, long P, int WM, int C4, int WZ) {
    if (dt != SOL_BF16 || WM != 256 || (WZ != 256 && WZ != 512) || C4 % 128 != 0 || C4 < 128 || C4 > 1024) return false;
    if (P <= 0) return false;
    return (double)P * C4 * 2.0 < 2147483648.0;
}

sol_status launch_conv_xr(const XrLaunch &b, hipStream_t st) {
    SOL_REQUIRE(xr_kernel_applies(SOL_BF16, b.P, b.WM, b.C4, b.WZ), SOL_ERR_UNSUPPORTED, "fused expand-reduce pair: unsupported shape");
    XrArgs a;
    a.t = b.t; a.r = b.r; a.y = b.y; a.z = b.z; a.w3 = b.w3; a.w1 = b.w1;
    a.s3 = b.s3; a.h3 = b.h3; a.s1 = b.s1; a.h1 = b.h1;
    a.P = (int)b.P; a.C4 = b.C4;
    a.ntiles = (a.P + 63) / 64;
    const int grid = ((a.ntiles + 7) / 8) * 8;
    if (b.WZ == 256) hipLaunchKernelGGL((conv_xr_kernel<256, 256, 6>), dim3(grid), dim3(512), 0, st, a);
    else hipLaunchKernelGGL((conv_xr_kernel<256, 512, 6>), dim3(grid), dim3(512), 0, st, a);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

}  // namespace sol

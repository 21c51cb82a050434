// Fused stride-2 convolutions over 3-channel inputs (network stems: 7x7 pad 3 of the ResNet-shaped lists, 3x3 of
// the depthwise-separable chain), bf16.  The text below describes the 7x7 case; a 3x3 filter pads each filter
// row to 16 reduction elements instead of 32.
//
// With Cin = 3 the reduction index (r, s, c) has no 16-byte-contiguous runs in NHWC, so the generic
// implicit GEMM has to gather single elements.  Here a workgroup instead stages the input patch of
// an 8 x 16 block of output pixels in LDS, widened to 4 channels per pixel (8 bytes, channel 3 = 0).
// For a fixed filter row r the taps (s, c) of one output pixel are then 7 x 4 contiguous elements,
// padded to 32: the reduction becomes 7 rows x 32 = 224 elements, and every MFMA fragment (8
// consecutive reduction elements of one pixel) is one aligned 16-byte LDS read.  The weights are
// re-laid-out once per workgroup into the same padded order (zeros at s = 7 and c = 3), and the
// workgroup then walks many tiles (persistent grid), so that cost is paid once.
#include "conv_common.h"
#include <type_traits>

namespace sol {

struct StemRowOffset {   // same map as StemRows for a block that lies inside the image, as an element offset
    unsigned base, wo, cout;     // base: offset of the block's pixel (p0, q0)
    __device__ __forceinline__ unsigned operator()(int r) const { return base + ((unsigned)(r >> 4) * wo + (unsigned)(r & 15)) * cout; }
};

struct StemRows {   // tile row (py*16+px) of the 8x16 output block -> output pixel index
    int n, p0, q0, Ho, Wo;
    __device__ __forceinline__ long operator()(int m) const {
        const int p = p0 + (m >> 4), q = q0 + (m & 15);
        return (p < Ho && q < Wo) ? ((long)n * Ho + p) * Wo + q : -1L;
    }
};

constexpr int STEM_TH = 8, STEM_TW = 16;

// R x S filter, NC blocks of 32 output channels
template <int R, int S, int NC>
__global__ void __launch_bounds__(256) conv_stem_kernel(const ConvArgs a, int tiles_h, int tiles_w, int ntiles) {
    constexpr int KROW = S * 4 <= 16 ? 16 : 32;                          // reduction elements per filter row (S x 4, padded)
    constexpr int STEM_IH = 2 * (STEM_TH - 1) + R;                       // patch extent ...
    constexpr int STEM_IW = 2 * STEM_TW + KROW / 4 - 2;                  // ... incl. the zero columns the row padding reads
    constexpr int COLS = 2 * (STEM_TW - 1) + S;                          // columns that hold image data
    constexpr int STEM_WROW = R * KROW + 8;                              // padded weight row (bank spread)
    __shared__ __align__(16) bf16_t wl[NC * 32 * STEM_WROW];            // 7x7, 64 channels: 29.0 KB
    __shared__ __align__(16) bf16_t xl[2][STEM_IH * STEM_IW * 4];       //  2 x 6.4 KB: the next tile's patch lands while this one is read
    __shared__ __align__(16) float strip[4 * 32 * (NC * 32 + 4)];       // 34.0 KB epilogue transposer

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bf16_t *__restrict__ xg = static_cast<const bf16_t *>(a.x);
    const bf16_t *__restrict__ wg = static_cast<const bf16_t *>(a.w);

    const int lr = lane & 31, lh = lane >> 5;
    const int py = 2 * wave + (lr >> 4), px = lr & 15;                   // this lane's output pixel in the block
    const unsigned xbase = ((2 * py) * STEM_IW + 2 * px) * 8;            // its patch origin, bytes
    f32x16_t acc[NC][1];
    const Affine8 aff = load_affine<NC>(a, lane, 0);

    // Input patch of a tile: STEM_IH x COLS pixels, 3 channels each, NP pixels per thread.
    constexpr int NPIX = STEM_IH * COLS, NP = (NPIX + 255) / 256;
    uint2 pv[NP];
    int rel[NP], pih[NP], piw[NP];                // this thread's patch pixels: element offset from the patch origin, row, column
#pragma unroll
    for (int i = 0; i < NP; i++) {
        const int e = tid + i * 256;
        pih[i] = e < NPIX ? e / COLS : -(1 << 20);                       // past the patch: fails every bounds check
        piw[i] = e % COLS;
        rel[i] = (pih[i] * a.W + piw[i]) * 3;
    }
    auto load_patch = [&](int tile) {             // global -> registers (issued one tile ahead); 32-bit element offsets
        const int tw = tile % tiles_w, t2 = tile / tiles_w;
        const int th = t2 % tiles_h, n = t2 / tiles_h;
        const int gh0 = 2 * th * STEM_TH - a.ph, gw0 = 2 * tw * STEM_TW - a.pw;
        const int base = ((n * a.H + gh0) * a.W + gw0) * 3;
#pragma unroll
        for (int i = 0; i < NP; i++) {
            pv[i] = make_uint2(0, 0);
            if ((unsigned)(gh0 + pih[i]) < (unsigned)a.H && (unsigned)(gw0 + piw[i]) < (unsigned)a.W) {
                const bf16_t *p = xg + (base + rel[i]);
                pv[i].x = (uint32_t)p[0] | ((uint32_t)p[1] << 16);
                pv[i].y = (uint32_t)p[2];
            }
        }
    };
    auto store_patch = [&](int buf) {             // registers -> LDS, widened to 4 channels
#pragma unroll
        for (int i = 0; i < NP; i++) {
            const int e = tid + i * 256;
            if (e < NPIX) {
                const int ih = e / COLS, iw = e % COLS;
                *reinterpret_cast<uint2 *>(&xl[buf][(ih * STEM_IW + iw) * 4]) = pv[i];
            }
        }
    };

    // Prologue, all of its memory latencies overlapped: first patch and affine constants (above) are in flight while
    // the weights are fetched.  Packed weights [k][(r*S+s)*3+c] -> LDS [k][r*KROW + s*4 + c], zero at s >= S and
    // c = 3: the packed rows are first copied as they are, by LDS DMA with every load in flight at once, into the
    // (still unused) epilogue transposer; the re-layout then runs LDS to LDS, one (k, r) filter row per thread and
    // trip.  (A gather straight from global memory costs one exposed round trip per element and used to take longer
    // than all the tiles of a workgroup together.)  The 8 pad elements that end each LDS row are never read.
    if ((int)blockIdx.x < ntiles) load_patch(blockIdx.x);
    {
        // Kp <= 256: at most NC * 16 KB, as NC * 4 DMA instructions of 1 KB per wave; chunks past the last row read zeros
        const __amdgpu_buffer_rsrc_t wr = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(wg), 0, a.Cout * a.Kp * 2, 0x00020000);
        unsigned char *stage = reinterpret_cast<unsigned char *>(strip);
#pragma unroll
        for (int j = 0; j < NC * 4; j++)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(wr, (__attribute__((address_space(3))) void *)(stage + (j * 4 + wave) * 1024), 16,
                                                     ((j * 4 + wave) * 64 + lane) * 16, 0, 0, 0);
    }
    static_assert(STEM_IW % 2 == 0, "patch buffers are whole 16-byte units");
    for (int i = tid; i < STEM_IH * STEM_IW; i += 256)                   // incl. the never-written pad columns
        reinterpret_cast<uint4 *>(&xl[0][0])[i] = make_uint4(0, 0, 0, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);                                  // vmcnt(0): weights staged, patch and constants here
    __syncthreads();                                                     // ... for every wave; zero fill done
    {
        const bf16_t *raw = reinterpret_cast<const bf16_t *>(strip);
        for (int i = tid; i < NC * 32 * R; i += 256) {
            const int k = i / R, r = i % R;
            __align__(16) bf16_t row[KROW];
#pragma unroll
            for (int j = 0; j < KROW; j++) row[j] = 0;
            if (k < a.Cout) {
#pragma unroll
                for (int j = 0; j < S * 3; j++) row[(j / 3) * 4 + j % 3] = raw[k * a.Kp + r * S * 3 + j];
            }
#pragma unroll
            for (int j = 0; j < KROW / 8; j++)
                *reinterpret_cast<uint4 *>(&wl[k * STEM_WROW + r * KROW + j * 8]) = *reinterpret_cast<const uint4 *>(&row[j * 8]);
        }
    }
    store_patch(0);
    // (the barrier that opens the first tile publishes wl and the patch, and orders the staging reads above before
    // any epilogue write to the transposer)

    // Wait bookkeeping: the compiler derives every vmcnt wait itself, and where paths join it assumes the worst of
    // them.  So everything loaded before the loop (affine constants, first patch) is drained in the prologue; inside the loop
    // a patch is written to LDS at the END of the iteration that issued its loads; and the loop exists twice, so
    // that the common one (every block inside the image, all channels, no residual) is straight-line code in which
    // the only memory operations younger than the patch loads are the block's 2 * NC output stores: those stay in
    // flight across the wait instead of stalling the next tile.  The explicit waits in the loop only tell the
    // compiler, at a point every lane passes, what it would otherwise have to assume at the next join; it still
    // adds any wait it needs itself.
    using namespace lds_pipe;
    constexpr int NKS = R * KROW / 16, DEPTH = 2;
    static_assert(sizeof(strip) >= NC * 16384, "weight staging area");
    static_assert(NKS >= DEPTH, "pipeline deeper than the reduction");
    u32x4_t fb[DEPTH + 1], fa[DEPTH + 1][NC];
    const unsigned aw = lds_addr(wl) + (lr * STEM_WROW + lh * 8) * 2;
    auto issue_step = [&](auto KS, unsigned ax) {
        constexpr int ks = decltype(KS)::value, slot = ks % (DEPTH + 1);
        lds_read16<((ks / (KROW / 16)) * STEM_IW + (ks % (KROW / 16)) * 4) * 8>(fb[slot], ax);
        static_for<NC>([&](auto I) { lds_read16<(decltype(I)::value * 32 * STEM_WROW + ks * 16) * 2>(fa[slot][decltype(I)::value], aw); });
    };

    auto run_tiles = [&](auto interior_tag) {
        constexpr bool INTERIOR = decltype(interior_tag)::value;
        int cur = 0;
        for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x, cur ^= 1) {
            const int tw = tile % tiles_w, t2 = tile / tiles_w;
            const int th = t2 % tiles_h, n = t2 / tiles_h;
            const int p0 = th * STEM_TH, q0 = tw * STEM_TW;
            const bool more = tile + (int)gridDim.x < ntiles;
            __syncthreads();                                             // xl[cur] written; xl[cur ^ 1] no longer read
            if (more) load_patch(tile + gridDim.x);                      // in flight under the MFMAs and the epilogue
#pragma unroll
            for (int i = 0; i < NC; i++)
#pragma unroll
                for (int e = 0; e < 16; e++) acc[i][0][e] = 0.f;
            // Reduction step ks covers 16 elements of filter row r = ks / (KROW / 16): 8 per lane half, i.e. patch
            // pixels s0, s0 + 1 with s0 = (ks % (KROW / 16)) * 4 + 2 * lh.  The fragment reads are issued by hand
            // DEPTH steps ahead of the MFMAs that consume them (left to itself the compiler issues them just in
            // time and every step waits out a full LDS round trip).
            const unsigned ax = lds_addr(xl[cur]) + xbase + lh * 16;
            static_for<DEPTH>([&](auto KS) { issue_step(KS, ax); });
            static_for<NKS>([&](auto KS) {
                constexpr int ks = decltype(KS)::value, slot = ks % (DEPTH + 1);
                if constexpr (ks + DEPTH < NKS) issue_step(std::integral_constant<int, ks + DEPTH>{}, ax);
                wait_lgkmcnt<(ks + DEPTH < NKS ? DEPTH : NKS - 1 - ks) * (1 + NC)>();
                landed(fb[slot]);
#pragma unroll
                for (int i = 0; i < NC; i++) {
                    landed(fa[slot][i]);
                    Mma<bf16_t>::run(acc[i][0], fa[slot][i], fb[slot]);
                }
            });
            ResidualRegs<bf16_t, 1, NC> resregs;
            resregs.on = false;
            if constexpr (INTERIOR) {                                    // branch-free epilogue
                const int pw = p0 + 2 * wave;     // first output row of this wave's 32 tile rows
                const StemRowOffset ro{(unsigned)(((n * a.Ho + pw) * a.Wo + q0) * (NC * 32)), (unsigned)a.Wo, (unsigned)(NC * 32)};
                conv_epilogue_interior<bf16_t, 1, NC, false>(a, acc, strip, wave, lane, 0, aff, resregs, ro);
                __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * NC));           // vmcnt(2 * NC), outside the lane-masked regions below
            } else {
                const StemRows rows{n, p0, q0, a.Ho, a.Wo};
                prefetch_residual<bf16_t, 1, NC>(a, lane, wave * 32, 0, rows, resregs);
                conv_epilogue<bf16_t, 1, NC>(a, acc, strip, wave, lane, wave * 32, 0, aff, rows, resregs);
                __builtin_amdgcn_s_waitcnt(0x0F70);
            }
            if (more) store_patch(cur ^ 1);
        }
    };
    if (a.Ho % STEM_TH == 0 && a.Wo % STEM_TW == 0 && a.Cout == NC * 32 && a.res == nullptr)
        run_tiles(std::true_type{});
    else
        run_tiles(std::false_type{});
}

bool stem_kernel_applies(const ConvArgs &a, int dt) {
    const bool k7 = a.R == 7 && a.S == 7, k3 = a.R == 3 && a.S == 3;
    return dt == SOL_BF16 && a.C == 3 && (k7 || k3) && a.sh == 2 && a.sw == 2 && a.ph >= 0 && a.ph < a.R && a.pw >= 0 && a.pw < a.S &&
           a.Cout <= 64 && a.pool == 0 && (long)a.N * a.H * a.W * 3 < (1L << 31) &&   // the patch loader uses 32-bit offsets
           a.Kp % 8 == 0 && a.Kp <= 256;   // the packed rows are staged whole in the transposer: 17 KB per 32 channels
}

sol_status launch_conv_stem(const ConvArgs &a, hipStream_t st) {
    const int tiles_h = ceil_div(a.Ho, STEM_TH), tiles_w = ceil_div(a.Wo, STEM_TW);
    const int ntiles = a.N * tiles_h * tiles_w;
    const int grid = ntiles < 512 ? ntiles : 512;                        // 2 persistent workgroups per CU
    if (a.R == 7 && a.Cout > 32)
        hipLaunchKernelGGL((conv_stem_kernel<7, 7, 2>), dim3(grid), dim3(256), 0, st, a, tiles_h, tiles_w, ntiles);
    else if (a.R == 7)
        hipLaunchKernelGGL((conv_stem_kernel<7, 7, 1>), dim3(grid), dim3(256), 0, st, a, tiles_h, tiles_w, ntiles);
    else if (a.Cout > 32)
        hipLaunchKernelGGL((conv_stem_kernel<3, 3, 2>), dim3(grid), dim3(256), 0, st, a, tiles_h, tiles_w, ntiles);
    else
        hipLaunchKernelGGL((conv_stem_kernel<3, 3, 1>), dim3(grid), dim3(256), 0, st, a, tiles_h, tiles_w, ntiles);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

}  // namespace sol

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

struct StemRowOffset {   // same map as StemRows as an element offset; rows past the image's last row / column are not stored
    unsigned base, wo, cout;     // base: offset of the wave's first pixel; cout: elements between pixels
    int hleft, wleft;            // output rows / columns from that pixel to the image border
    __device__ __forceinline__ unsigned operator()(int r) const { return base + ((unsigned)(r >> 4) * wo + (unsigned)(r & 15)) * cout; }
    __device__ __forceinline__ bool valid(int r) const { return (r >> 4) < hleft && (r & 15) < wleft; }
    __device__ __forceinline__ unsigned lane_base(int lane_row) const { return (unsigned)lane_row; }      // the map is not linear in the row: kept as the row
    __device__ __forceinline__ unsigned at(unsigned lb, int r) const { return (*this)((int)lb + r); }
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
    // that the common one (all NC * 32 channels, no residual; rows past the image border are masked) is straight-line code in which
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
                const StemRowOffset ro{(unsigned)(((n * a.Ho + pw) * a.Wo + q0) * a.ldy), (unsigned)a.Wo, (unsigned)a.ldy, a.Ho - pw, a.Wo - q0};
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
    if (a.Cout == NC * 32 && a.res == nullptr)       // ragged image extents are handled by the row mask of the fast epilogue
        run_tiles(std::true_type{});
    else
        run_tiles(std::false_type{});
}

// ---- 7x7 stride-2 stem + ReLU + 3x3 stride-2 pad-1 max pool in one kernel ---------------------------------
// The stem's output is the largest tensor of a ResNet-shaped list and its only consumer is the max pool behind
// it, so the pair is run depth-first: a workgroup computes the 15 x 17 convolution pixels under a 7 x 8 block of
// pool outputs (the one-pixel overlap between neighbouring blocks is recomputed: 255 pixels for 56 x 4), applies
// the affine map and the ReLU, parks the block in LDS as bf16 and takes the 3x3 maxima from there.  Only the
// pooled tensor reaches memory.  Rounding to bf16 before the maximum is what the two-kernel path does too
// (rounding is monotonic, so the results are identical).  After the ReLU every value is >= +0, so bf16 bit
// patterns order like unsigned integers (packed 16-bit maxima) and convolution pixels outside the image, which
// the pool must ignore, are stored as 0: every window holds at least one real pixel.
constexpr int SP_PH = 7, SP_PW = 8;                      // pool outputs per block
constexpr int SP_CH = 2 * SP_PH + 1, SP_CW = 2 * SP_PW + 1;   // convolution pixels under them: 15 x 17
constexpr int SP_R = 7, SP_KROW = 32;
constexpr int SP_IH = 2 * (SP_CH - 1) + SP_R;            // 35 input rows
constexpr int SP_COLS = 2 * (SP_CW - 1) + SP_R;          // 39 input columns with data
constexpr int SP_IW = 2 * SP_CW + SP_KROW / 4 - 2;       // 40: incl. the zero column the row padding reads
constexpr int SP_WROW = SP_R * SP_KROW + 8;
constexpr int SP_PITCH = 72;                             // bf16 elements per parked pixel (64 + 8: bank spread)

typedef __attribute__((ext_vector_type(8))) unsigned short u16x8_t;

__global__ void __launch_bounds__(256) conv_stem_pool_kernel(const ConvArgs a, int tiles_h, int tiles_w, int ntiles) {
    using namespace lds_pipe;
    constexpr int R = SP_R, S = 7, KROW = SP_KROW, NC = 2;
    __shared__ __align__(16) bf16_t wl[NC * 32 * SP_WROW];              // 29.0 KB
    __shared__ __align__(16) bf16_t xl[SP_IH * SP_IW * 4];              // 10.9 KB
    __shared__ __align__(16) bf16_t ct[256 * SP_PITCH];                 // 36.0 KB parked block; weight staging before the first tile
    __shared__ __align__(16) float aff[2][64];                          // scale, shift
    static_assert(sizeof(ct) >= NC * 16384, "weight staging area");
    static_assert((SP_IH * SP_IW) % 2 == 0, "patch buffer is whole 16-byte units");

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 31, lh = lane >> 5;
    const bf16_t *__restrict__ xg = static_cast<const bf16_t *>(a.x);
    const bf16_t *__restrict__ wg = static_cast<const bf16_t *>(a.w);
    bf16_t *__restrict__ yg = static_cast<bf16_t *>(a.y);

    // input patch of a block: SP_IH x SP_COLS pixels of 3 channels, NP per thread, 32-bit element offsets
    constexpr int NPIX = SP_IH * SP_COLS, NP = (NPIX + 255) / 256;
    uint2 pv[NP];
    int rel[NP], pih[NP], piw[NP];
#pragma unroll
    for (int i = 0; i < NP; i++) {
        const int e = tid + i * 256;
        pih[i] = e < NPIX ? e / SP_COLS : -(1 << 20);                    // past the patch: fails every bounds check
        piw[i] = e % SP_COLS;
        rel[i] = (pih[i] * a.W + piw[i]) * 3;
    }
    auto tile_origin = [&](int tile, int &n, int &py0, int &px0) {
        const int tw = tile % tiles_w, t2 = tile / tiles_w;
        n = t2 / tiles_h; py0 = (t2 % tiles_h) * SP_PH; px0 = tw * SP_PW;
    };
    auto load_patch = [&](int tile) {
        int n, py0, px0;
        tile_origin(tile, n, py0, px0);
        // pool row py covers convolution rows 2 py - 1 .. 2 py + 1; convolution row q covers input rows 2 q - ph ..
        const int gh0 = 2 * (2 * py0 - 1) - a.ph, gw0 = 2 * (2 * px0 - 1) - a.pw;
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
    auto store_patch = [&]() {
#pragma unroll
        for (int i = 0; i < NP; i++) {
            const int e = tid + i * 256;
            if (e < NPIX) *reinterpret_cast<uint2 *>(&xl[((e / SP_COLS) * SP_IW + e % SP_COLS) * 4]) = pv[i];
        }
    };

    // prologue: first patch, weights (staged by DMA in the parked-block area, re-laid-out LDS to LDS), constants
    if ((int)blockIdx.x < ntiles) load_patch(blockIdx.x);
    {
        const __amdgpu_buffer_rsrc_t wr = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(wg), 0, a.Cout * a.Kp * 2, 0x00020000);
        unsigned char *stage = reinterpret_cast<unsigned char *>(ct);
#pragma unroll
        for (int j = 0; j < NC * 4; j++)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(wr, (__attribute__((address_space(3))) void *)(stage + (j * 4 + wave) * 1024), 16,
                                                     ((j * 4 + wave) * 64 + lane) * 16, 0, 0, 0);
    }
    if (tid < 128) aff[tid >> 6][tid & 63] = tid < 64 ? (a.scale ? a.scale[tid] : 1.f) : (a.shift ? a.shift[tid - 64] : 0.f);
    for (int i = tid; i < SP_IH * SP_IW / 2; i += 256) reinterpret_cast<uint4 *>(xl)[i] = make_uint4(0, 0, 0, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);                                  // vmcnt(0)
    __syncthreads();
    {
        const bf16_t *raw = reinterpret_cast<const bf16_t *>(ct);
        for (int i = tid; i < NC * 32 * R; i += 256) {
            const int k = i / R, r = i % R;
            __align__(16) bf16_t row[KROW];
#pragma unroll
            for (int j = 0; j < KROW; j++) row[j] = 0;
#pragma unroll
            for (int j = 0; j < S * 3; j++) row[(j / 3) * 4 + j % 3] = raw[k * a.Kp + r * S * 3 + j];
#pragma unroll
            for (int j = 0; j < KROW / 8; j++)
                *reinterpret_cast<uint4 *>(&wl[k * SP_WROW + r * KROW + j * 8]) = *reinterpret_cast<const uint4 *>(&row[j * 8]);
        }
    }
    store_patch();

    // this lane's two convolution pixels (one per 32-pixel block of its wave): m = cy * 17 + cx; the 256th is a duplicate
    int cy[2], cx[2];
    unsigned ax[2], ctoff[2];
#pragma unroll
    for (int jb = 0; jb < 2; jb++) {
        const int m = min((2 * wave + jb) * 32 + lr, SP_CH * SP_CW - 1);
        cy[jb] = m / SP_CW; cx[jb] = m % SP_CW;
        ax[jb] = lds_addr(xl) + ((2 * cy[jb]) * SP_IW + 2 * cx[jb]) * 8 + lh * 16;
        ctoff[jb] = ((2 * wave + jb) * 32 + lr) * SP_PITCH + 4 * lh;
    }
    const unsigned aw = lds_addr(wl) + (lr * SP_WROW + lh * 8) * 2;
    constexpr int NKS = R * KROW / 16, DEPTH = 2;
    u32x4_t fb[DEPTH + 1][2], fa[DEPTH + 1][NC];
    auto issue_step = [&](auto KS) {
        constexpr int ks = decltype(KS)::value, slot = ks % (DEPTH + 1);
        constexpr int xoff = ((ks / (KROW / 16)) * SP_IW + (ks % (KROW / 16)) * 4) * 8;
        lds_read16<xoff>(fb[slot][0], ax[0]);
        lds_read16<xoff>(fb[slot][1], ax[1]);
        static_for<NC>([&](auto I) { lds_read16<(decltype(I)::value * 32 * SP_WROW + ks * 16) * 2>(fa[slot][decltype(I)::value], aw); });
    };
    f32x16_t acc[NC][2];

    for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        int n, py0, px0;
        tile_origin(tile, n, py0, px0);
        const bool more = tile + (int)gridDim.x < ntiles;
        __syncthreads();                                                 // patch and weights written; parked block no longer read
        if (more) load_patch(tile + gridDim.x);                          // lands under the MFMAs
#pragma unroll
        for (int i = 0; i < NC; i++)
#pragma unroll
            for (int jb = 0; jb < 2; jb++)
#pragma unroll
                for (int e = 0; e < 16; e++) acc[i][jb][e] = 0.f;
        static_for<DEPTH>([&](auto KS) { issue_step(KS); });
        static_for<NKS>([&](auto KS) {
            constexpr int ks = decltype(KS)::value, slot = ks % (DEPTH + 1);
            if constexpr (ks + DEPTH < NKS) issue_step(std::integral_constant<int, ks + DEPTH>{});
            wait_lgkmcnt<(ks + DEPTH < NKS ? DEPTH : NKS - 1 - ks) * (2 + NC)>();
            landed(fb[slot][0]); landed(fb[slot][1]);
#pragma unroll
            for (int i = 0; i < NC; i++) {
                landed(fa[slot][i]);
                Mma<bf16_t>::run(acc[i][0], fa[slot][i], fb[slot][0]);
                Mma<bf16_t>::run(acc[i][1], fa[slot][i], fb[slot][1]);
            }
        });
        // accumulator register e of lane l: channel 32 i + 8 (e / 4) + 4 (l / 32) + e % 4 of pixel l % 32
#pragma unroll
        for (int jb = 0; jb < 2; jb++) {
            const int q = 2 * py0 - 1 + cy[jb], p = 2 * px0 - 1 + cx[jb];
            const bool real = (unsigned)q < (unsigned)a.Ho && (unsigned)p < (unsigned)a.Wo;
#pragma unroll
            for (int i = 0; i < NC; i++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    const int c = 32 * i + 8 * g + 4 * lh;
                    const float4 sc = *reinterpret_cast<const float4 *>(&aff[0][c]), sf = *reinterpret_cast<const float4 *>(&aff[1][c]);
                    float v0 = acc[i][jb][4 * g + 0] * sc.x + sf.x, v1 = acc[i][jb][4 * g + 1] * sc.y + sf.y;
                    float v2 = acc[i][jb][4 * g + 2] * sc.z + sf.z, v3 = acc[i][jb][4 * g + 3] * sc.w + sf.w;
                    v0 = __builtin_fmaxf(v0, 0.f); v1 = __builtin_fmaxf(v1, 0.f); v2 = __builtin_fmaxf(v2, 0.f); v3 = __builtin_fmaxf(v3, 0.f);   // one v_max each; a NaN becomes 0
                    uint2 pk = make_uint2(pack_bf16x2(v0, v1), pack_bf16x2(v2, v3));
                    if (!real) pk = make_uint2(0, 0);
                    *reinterpret_cast<uint2 *>(&ct[ctoff[jb] + 32 * i + 8 * g]) = pk;
                }
        }
        __syncthreads();                                                 // block parked; nobody reads the patch any more
        if (more) store_patch();
        // 56 pool outputs x 8 chunks of 8 channels
        for (int t = tid; t < SP_PH * SP_PW * 8; t += 256) {
            const int chunk = t & 7, o = t >> 3, oy = o / SP_PW, ox = o % SP_PW;
            const int py = py0 + oy, px = px0 + ox;
            if (py >= a.Hy || px >= a.Wy) continue;
            const bf16_t *base = &ct[((2 * oy) * SP_CW + 2 * ox) * SP_PITCH + chunk * 8];
            u16x8_t m = *reinterpret_cast<const u16x8_t *>(base);
#pragma unroll
            for (int d = 1; d < 9; d++)
                m = __builtin_elementwise_max(m, *reinterpret_cast<const u16x8_t *>(base + ((d / 3) * SP_CW + d % 3) * SP_PITCH));
            *reinterpret_cast<u16x8_t *>(yg + (((long)n * a.Hy + py) * a.Wy + px) * 64 + chunk * 8) = m;
        }
    }
}

// 7x7 stride-2 stem with 64 output channels, ReLU, no residual, followed by a 3x3 stride-2 pad-1 max pool
bool stem_pool_applies(const ConvArgs &a, int dt, const sol_pool_desc &p) {
    return dt == SOL_BF16 && a.C == 3 && a.R == 7 && a.S == 7 && a.sh == 2 && a.sw == 2 && a.ph >= 0 && a.ph < 7 && a.pw >= 0 && a.pw < 7 &&
           a.Cout == 64 && a.act == SOL_ACT_RELU && a.res == nullptr && (long)a.N * a.H * a.W * 3 < (1L << 31) && a.Kp % 8 == 0 &&
           a.Kp <= 256 && p.kind == SOL_POOL_MAX && p.kh == 3 && p.kw == 3 && p.sh == 2 && p.sw == 2 && p.ph == 1 && p.pw == 1;
}

sol_status launch_conv_stem_pool(const ConvArgs &a, hipStream_t st) {
    const int tiles_h = ceil_div(a.Hy, SP_PH), tiles_w = ceil_div(a.Wy, SP_PW);
    const int ntiles = a.N * tiles_h * tiles_w;
    if (ntiles == 0) return SOL_OK;
    const int grid = ntiles < 512 ? ntiles : 512;                        // 2 persistent workgroups per CU
    hipLaunchKernelGGL(conv_stem_pool_kernel, dim3(grid), dim3(256), 0, st, a, tiles_h, tiles_w, ntiles);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
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

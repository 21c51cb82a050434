// Projection shortcut and the 1x1 convolution it is added to, as one kernel (bf16, both reductions 64 channels):
//
//     out[m][k] = act( scale3[k] * sum_c y2[m][c] w3[k][c] + shift3[k] + scale_d[k] * sum_c x[m][c] wd[k][c] + shift_d[k] )
//
// In the first bottleneck of a ResNet-shaped list the shortcut is a 1x1 convolution of the block input whose only
// reader is the residual add of the block's last 1x1 convolution.  Run as two layers, its output -- as large as the
// block output, the largest tensor of the stage -- is written once and read back once.  Here a workgroup fetches
// the two pixel tiles and the two weight tiles of a 128 x 128 output block (four 16 KB operands, every DMA in flight
// at once), runs both contractions into accumulators of their own, combines them in fp32 in the accumulator
// layout and hands the sum to the usual branch-free epilogue with an identity affine map.  The shortcut is
// never rounded to bf16, which the two-layer path does when it stores it: results differ from that path by at
// most one bf16 rounding of the shortcut term (well inside the tolerance of the library).
// Overlap of loads, MFMAs and stores comes from two resident workgroups per CU; the job is bound by HBM.
#include "conv_common.h"
#include <type_traits>

namespace sol {

constexpr int PR_BP = 128, PR_BC = 128, PR_ROWB = 128;           // output block; bytes of reduction per row (64 bf16)
constexpr int PR_OPB = 128 * PR_ROWB;                            // bytes of one operand tile

__global__ void __launch_bounds__(256, 2) conv_pair_k64_kernel(const ConvArgs a, const void *x2v, const void *w2v,
                                                            const float *__restrict__ scale2, const float *__restrict__ shift2) {
    using namespace lds_pipe;
    constexpr int TP = 2, TC = 2, KS = PR_ROWB / 32;
    __shared__ __align__(1024) unsigned char lds[4 * PR_OPB];   // y2 | w3 | x | wd tiles; later the epilogue strips
    __shared__ __align__(16) float chan[3][PR_BC];               // scale3, scale_d, shift3 + shift_d of the block's channels
    static_assert(4 * 32 * (TC * 32 + 4) * 4 <= 4 * PR_OPB, "epilogue strips fit in the operand area");

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wp = wave & 1, wc = wave >> 1;
    const int xcd = (int)(blockIdx.x & 7);
    const int tile = xcd * ((a.ntiles + 7) >> 3) + (int)(blockIdx.x >> 3);   // an XCD takes a contiguous run of blocks
    if (tile >= a.ntiles) return;
    const int p0 = (tile / a.ntc) * PR_BP, c0 = (tile % a.ntc) * PR_BC;

    // operand o: 0 = y2 (a.x), 1 = w3 (a.w), 2 = x (x2v), 3 = wd (w2v); rows past the tensors read zeros
    const unsigned pbytes = (unsigned)a.P * 64u * 2u, wbytes = (unsigned)a.Cout * (unsigned)a.Kp * 2u;
    const __amdgpu_buffer_rsrc_t rs[4] = {
        __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.x), 0, (int)pbytes, 0x00020000),
        __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.w), 0, (int)wbytes, 0x00020000),
        __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(x2v), 0, (int)pbytes, 0x00020000),
        __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(w2v), 0, (int)wbytes, 0x00020000)};
    const int lslot = lane & 7, lrow = lane >> 3;              // a 1 KB DMA segment = 8 rows x 8 slots of 16 bytes
    auto swz = [](int row) { return (row >> 1) & 7; };
#pragma unroll
    for (int o = 0; o < 4; o++)
#pragma unroll
        for (int i = 0; i < 4; i++) {                           // 16 segments per operand, 4 per wave
            const int seg = i * 4 + wave, row = seg * 8 + lrow;
            const bool pix = (o & 1) == 0;
            const int g = (pix ? p0 : c0) + row;
            const bool ok = g < (pix ? a.P : a.Cout);
            const unsigned off = ok ? (unsigned)g * (pix ? 128u : (unsigned)a.Kp * 2u) + (unsigned)((lslot ^ swz(row)) << 4) : 0xffffffffu;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs[o], (__attribute__((address_space(3))) void *)(lds + o * PR_OPB + seg * 1024), 16,
                                                     off, 0, 0, 0);
        }
    // per-channel constants: fetched by every thread (uniform instruction count per wave), parked in LDS only after
    // the contractions -- a store to LDS right here would make the compiler wait for everything issued above
    const int cc = min(c0 + (tid & (PR_BC - 1)), a.Cout - 1);
    const float k_s3 = a.scale ? a.scale[cc] : 1.f, k_sd = scale2 ? scale2[cc] : 1.f;
    const float k_h3 = a.shift ? a.shift[cc] : 0.f, k_hd = shift2 ? shift2[cc] : 0.f;   // first used behind the contractions

    f32x16_t acc3[TC][TP], accd[TC][TP];
#pragma unroll
    for (int i = 0; i < TC; i++)
#pragma unroll
        for (int j = 0; j < TP; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) { acc3[i][j][e] = 0.f; accd[i][j][e] = 0.f; }

    const int lr = lane & 31, lh = lane >> 5;
    const int fsw = swz(lr);                                    // tile row bases are multiples of 32
    // the first contraction starts when its two operands are here (8 of this wave's 16 DMA instructions; whatever else
    // is in flight is younger), the other two land under its MFMAs
    wait_vmcnt<8>();
    __builtin_amdgcn_s_barrier();     // bare barriers: a fence would drain the loads that are meant to stay in flight

    // The fragment reads are opaque statements: the compiler, which cannot tell the operands apart, would make every
    // LDS read wait for all outstanding DMA, also those of the operands the second contraction uses.
    auto contract = [&](f32x16_t (&acc)[TC][TP], const unsigned char *xt, const unsigned char *wt) {
        const unsigned ax = lds_addr(xt) + (wp * TP * 32 + lr) * PR_ROWB, aw = lds_addr(wt) + (wc * TC * 32 + lr) * PR_ROWB;
        // two fragment sets alternate: the reads of k-step ks + 1 fly under the MFMAs of k-step ks
        u32x4_t fa[2][TC], fb[2][TP];
        auto read_set = [&](auto SET, int ks) {
            constexpr int set = decltype(SET)::value;
            const unsigned so = (unsigned)(((2 * ks + lh) ^ fsw) << 4);
            static_for<TC>([&](auto I) { lds_read16<decltype(I)::value * 32 * PR_ROWB>(fa[set][decltype(I)::value], aw + so); });
            static_for<TP>([&](auto J) { lds_read16<decltype(J)::value * 32 * PR_ROWB>(fb[set][decltype(J)::value], ax + so); });
        };
        read_set(std::integral_constant<int, 0>{}, 0);
        static_for<KS>([&](auto KSI) {
            constexpr int ks = decltype(KSI)::value, cur = ks & 1;
            if constexpr (ks + 1 < KS) {
                read_set(std::integral_constant<int, cur ^ 1>{}, ks + 1);
                wait_lgkmcnt<TC + TP>();           // LDS returns in order: all but the newest TC + TP reads are done
            } else {
                wait_lgkmcnt<0>();
            }
            static_for<TC>([&](auto I) { landed(fa[cur][decltype(I)::value]); });
            static_for<TP>([&](auto J) { landed(fb[cur][decltype(J)::value]); });
#pragma unroll
            for (int i = 0; i < TC; i++)
#pragma unroll
                for (int j = 0; j < TP; j++) Mma<bf16_t>::run(acc[i][j], fa[cur][i], fb[cur][j]);
        });
    };
    contract(acc3, lds, lds + PR_OPB);
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    contract(accd, lds + 2 * PR_OPB, lds + 3 * PR_OPB);
    if (tid < PR_BC) { chan[0][tid] = k_s3; chan[1][tid] = k_sd; chan[2][tid] = k_h3 + k_hd; }
    __syncthreads();

    // accumulator register e of lane l: channel 32 i + 8 (e / 4) + 4 (l / 32) + e % 4 of the wave's block
#pragma unroll
    for (int i = 0; i < TC; i++)
#pragma unroll
        for (int g = 0; g < 4; g++) {
            const int c = wc * TC * 32 + 32 * i + 8 * g + 4 * lh;
            const float4 s3 = *reinterpret_cast<const float4 *>(&chan[0][c]), sd = *reinterpret_cast<const float4 *>(&chan[1][c]);
            const float4 sh = *reinterpret_cast<const float4 *>(&chan[2][c]);
#pragma unroll
            for (int j = 0; j < TP; j++) {
                acc3[i][j][4 * g + 0] = acc3[i][j][4 * g + 0] * s3.x + (accd[i][j][4 * g + 0] * sd.x + sh.x);
                acc3[i][j][4 * g + 1] = acc3[i][j][4 * g + 1] * s3.y + (accd[i][j][4 * g + 1] * sd.y + sh.y);
                acc3[i][j][4 * g + 2] = acc3[i][j][4 * g + 2] * s3.z + (accd[i][j][4 * g + 2] * sd.z + sh.z);
                acc3[i][j][4 * g + 3] = acc3[i][j][4 * g + 3] * s3.w + (accd[i][j][4 * g + 3] * sd.w + sh.w);
            }
        }
    Affine8 unit;
#pragma unroll
    for (int e = 0; e < 8; e++) { unit.sc[e] = 1.f; unit.sf[e] = 0.f; }
    ResidualRegs<bf16_t, TP, TC> none;
    none.on = false;
    __syncthreads();                                            // every wave is done with the operand tiles: they become strips
    conv_epilogue_auto<bf16_t, TP, TC>(a, acc3, reinterpret_cast<float *>(lds), wave, lane, p0 + wp * TP * 32, c0 + wc * TC * 32, unit,
                                       LinearRows{a.P}, none);
}

// The same pair for reductions of any multiple of 64 channels and a strided shortcut (the first bottleneck of the later
// stages: the shortcut reads every second pixel of the previous stage's output).  The reduction runs in chunks of 64
// channels -- first those of the main convolution, then those of the shortcut, each into its own accumulators --
// through two LDS stages of one pixel tile + one weight tile; the DMA of chunk c + 1 is in flight while chunk c is
// contracted, and two workgroups share a CU.
struct PairGeom {
    const void *x2, *w2;
    const float *scale2, *shift2;
    int H2, W2, K2, Kp2, stride;            // shortcut input extent, channels, packed row length, stride
};

__global__ void __launch_bounds__(256, 2) conv_pair_kernel(const ConvArgs a, const PairGeom g) {
    using namespace lds_pipe;
    constexpr int TP = 2, TC = 2, KS = PR_ROWB / 32, STG = 2 * PR_OPB;
    __shared__ __align__(1024) unsigned char lds[2 * STG];      // two stages of [pixel tile | weight tile]; later the strips
    __shared__ __align__(16) float chan[3][PR_BC];
    static_assert(4 * 32 * (TC * 32 + 4) * 4 <= 2 * STG, "epilogue strips fit in the stages");

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wp = wave & 1, wc = wave >> 1;
    const int xcd = (int)(blockIdx.x & 7);
    const int tile = xcd * ((a.ntiles + 7) >> 3) + (int)(blockIdx.x >> 3);
    if (tile >= a.ntiles) return;
    const int p0 = (tile / a.ntc) * PR_BP, c0 = (tile % a.ntc) * PR_BC;
    const int n3 = a.C / 64, nd = g.K2 / 64, nchunk = n3 + nd;
    // Each pixel tile walks the chunks of either reduction in a rotation of its own (the channel tiles of a pixel tile share one,
    // so they still meet at the same pixel rows): workgroups run in step, and with every tile at the same chunk all requests of
    // the moment fall on the same offset inside rows whose pitch is a large power of two.  Same terms, summed in an order that
    // depends on the tile index alone.  Worth 0.2 to 1 % of a ResNet-50-shaped pass, depending on the machine.
    const int off3 = (tile / a.ntc) % n3, offd = (tile / a.ntc) % nd;

    const __amdgpu_buffer_rsrc_t r_y = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.x), 0, (int)((unsigned)a.P * a.C * 2u), 0x00020000);
    const __amdgpu_buffer_rsrc_t r_w3 = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.w), 0, (int)((unsigned)a.Cout * a.Kp * 2u), 0x00020000);
    const __amdgpu_buffer_rsrc_t r_x = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(g.x2), 0,
                                                                         (int)((unsigned)a.N * g.H2 * g.W2 * g.K2 * 2u), 0x00020000);
    const __amdgpu_buffer_rsrc_t r_wd = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(g.w2), 0, (int)((unsigned)a.Cout * g.Kp2 * 2u), 0x00020000);

    // this lane's four rows of a pixel tile and of a weight tile: byte offset of the row's chunk 0, slot permuted; rows past
    // the tensors get an offset beyond every buffer (all buffers are below 2 GB) and read zeros
    const int lslot = lane & 7, lrow = lane >> 3;
    auto swz = [](int row) { return (row >> 1) & 7; };
    constexpr unsigned OOB = 0x80000000u;
    unsigned oy[4], ox[4], o3[4], od[4];
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const int row = (i * 4 + wave) * 8 + lrow;
        const unsigned sl = (unsigned)((lslot ^ swz(row)) << 4);
        const int m = p0 + row, co = c0 + row;
        oy[i] = ox[i] = o3[i] = od[i] = OOB;
        if (m < a.P) {
            int n, p, q;
            decode_pixel(a, m, n, p, q);
            oy[i] = (unsigned)m * (unsigned)a.C * 2u + sl;
            ox[i] = (unsigned)((n * g.H2 + p * g.stride) * g.W2 + q * g.stride) * (unsigned)g.K2 * 2u + sl;
        }
        if (co < a.Cout) {
            o3[i] = (unsigned)co * (unsigned)a.Kp * 2u + sl;
            od[i] = (unsigned)co * (unsigned)g.Kp2 * 2u + sl;
        }
    }
    // IDX-th of the 8 DMA instructions of this wave for chunk c of the concatenated reduction into stage buf (even: pixel rows,
    // odd: weight rows)
    auto issue_one = [&](auto IDX, bool main, unsigned col, int buf) {
        constexpr int idx = decltype(IDX)::value, i = idx >> 1;
        unsigned char *st = lds + buf * STG;
        const int seg = i * 4 + wave;
        if constexpr ((idx & 1) == 0)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(main ? r_y : r_x, (__attribute__((address_space(3))) void *)(st + seg * 1024), 16,
                                                     (main ? oy[i] : ox[i]) + col, 0, 0, 0);
        else
            __builtin_amdgcn_raw_ptr_buffer_load_lds(main ? r_w3 : r_wd, (__attribute__((address_space(3))) void *)(st + PR_OPB + seg * 1024),
                                                     16, (main ? o3[i] : od[i]) + col, 0, 0, 0);
    };
    // chunk c of the concatenated reduction: which operand pair, and the byte offset of its columns inside a row
    auto chunk_col = [&](int c, bool &main) {
        main = c < n3;
        int cr = main ? c + off3 : c - n3 + offd;
        if (cr >= (main ? n3 : nd)) cr -= main ? n3 : nd;
        return (unsigned)cr * 128u;
    };
    {
        bool main0;
        const unsigned col0 = chunk_col(0, main0);
        static_for<8>([&](auto I) { issue_one(I, main0, col0, 0); });
    }
    const int cc = min(c0 + (tid & (PR_BC - 1)), a.Cout - 1);
    const float k_s3 = a.scale ? a.scale[cc] : 1.f, k_sd = g.scale2 ? g.scale2[cc] : 1.f;
    const float k_h3 = a.shift ? a.shift[cc] : 0.f, k_hd = g.shift2 ? g.shift2[cc] : 0.f;   // first used behind the loop

    f32x16_t acc3[TC][TP], accd[TC][TP];
#pragma unroll
    for (int i = 0; i < TC; i++)
#pragma unroll
        for (int j = 0; j < TP; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) { acc3[i][j][e] = 0.f; accd[i][j][e] = 0.f; }

    const int lr = lane & 31, lh = lane >> 5;
    const int fsw = swz(lr);
    // between(k): called behind the MFMAs of k-step k.  The DMA instructions of the next chunk go out there, two per k-step:
    // a wave issues in order, and issued up front they would queue at the CU's address unit (about 18 cycles per
    // instruction, both workgroups' waves at once) with every wave's MFMAs waiting behind them
    auto contract = [&](f32x16_t (&acc)[TC][TP], unsigned stage, auto &&between) {
        const unsigned ax = stage + (wp * TP * 32 + lr) * PR_ROWB, aw = stage + PR_OPB + (wc * TC * 32 + lr) * PR_ROWB;
        // one fragment set here: a second set (reads of the next k-step under these MFMAs) pays in the 64-channel
        // kernel above, but with this kernel's per-lane gather offsets live it spills registers and runs slower
        static_for<KS>([&](auto KSI) {
            constexpr int ks = decltype(KSI)::value;
            const unsigned so = (unsigned)(((2 * ks + lh) ^ fsw) << 4);
            u32x4_t fa[TC], fb[TP];
            static_for<TC>([&](auto I) { lds_read16<decltype(I)::value * 32 * PR_ROWB>(fa[decltype(I)::value], aw + so); });
            static_for<TP>([&](auto J) { lds_read16<decltype(J)::value * 32 * PR_ROWB>(fb[decltype(J)::value], ax + so); });
            wait_lgkmcnt<0>();
            static_for<TC>([&](auto I) { landed(fa[decltype(I)::value]); });
            static_for<TP>([&](auto J) { landed(fb[decltype(J)::value]); });
#pragma unroll
            for (int i = 0; i < TC; i++)
#pragma unroll
                for (int j = 0; j < TP; j++) Mma<bf16_t>::run(acc[i][j], fa[i], fb[j]);
            between(KSI);
        });
    };
    const unsigned lbase = lds_addr(lds);
    for (int c = 0; c < nchunk; c++) {
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();                           // chunk c has landed for every wave, and every wave has contracted chunk c - 1
        const bool more = c + 1 < nchunk;          // workgroup-uniform
        bool mainn;
        const unsigned coln = chunk_col(c + 1, mainn);
        auto dma = [&](auto K) {
            constexpr int k = decltype(K)::value;
            static_assert(KS == 4, "8 DMA instructions over 4 k-steps");
            if (more) {
                issue_one(std::integral_constant<int, 2 * k>{}, mainn, coln, (c + 1) & 1);
                issue_one(std::integral_constant<int, 2 * k + 1>{}, mainn, coln, (c + 1) & 1);
            }
        };
        if (c < n3) contract(acc3, lbase + (c & 1) * STG, dma); else contract(accd, lbase + (c & 1) * STG, dma);
    }
    if (tid < PR_BC) { chan[0][tid] = k_s3; chan[1][tid] = k_sd; chan[2][tid] = k_h3 + k_hd; }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < TC; i++)
#pragma unroll
        for (int gq = 0; gq < 4; gq++) {
            const int c = wc * TC * 32 + 32 * i + 8 * gq + 4 * lh;
            const float4 s3 = *reinterpret_cast<const float4 *>(&chan[0][c]), sd = *reinterpret_cast<const float4 *>(&chan[1][c]);
            const float4 sh = *reinterpret_cast<const float4 *>(&chan[2][c]);
#pragma unroll
            for (int j = 0; j < TP; j++) {
                acc3[i][j][4 * gq + 0] = acc3[i][j][4 * gq + 0] * s3.x + (accd[i][j][4 * gq + 0] * sd.x + sh.x);
                acc3[i][j][4 * gq + 1] = acc3[i][j][4 * gq + 1] * s3.y + (accd[i][j][4 * gq + 1] * sd.y + sh.y);
                acc3[i][j][4 * gq + 2] = acc3[i][j][4 * gq + 2] * s3.z + (accd[i][j][4 * gq + 2] * sd.z + sh.z);
                acc3[i][j][4 * gq + 3] = acc3[i][j][4 * gq + 3] * s3.w + (accd[i][j][4 * gq + 3] * sd.w + sh.w);
            }
        }
    Affine8 unit;
#pragma unroll
    for (int e = 0; e < 8; e++) { unit.sc[e] = 1.f; unit.sf[e] = 0.f; }
    ResidualRegs<bf16_t, TP, TC> none;
    none.on = false;
    __syncthreads();
    conv_epilogue_auto<bf16_t, TP, TC>(a, acc3, reinterpret_cast<float *>(lds), wave, lane, p0 + wp * TP * 32, c0 + wc * TC * 32, unit,
                                       LinearRows{a.P}, none);
}

// a: the convolution that carries the residual (its x, w, scale, shift, y); both convolutions 1x1 stride 1 unpadded over
// 64 channels, a.res unused
bool pair_k64_applies(const ConvArgs &a, int dt) {
    return dt == SOL_BF16 && a.R == 1 && a.S == 1 && a.sh == 1 && a.sw == 1 && a.ph == 0 && a.pw == 0 && a.C == 64 && a.Kp == 64 &&
           a.pool == 0 && a.Cout % 8 == 0 && (double)a.P * a.ldy < 4294967296.0;
}

sol_status launch_conv_pair_k64(ConvArgs a, const void *x2, const void *w2, const float *scale2, const float *shift2, hipStream_t st);

// a: the main convolution (1x1 stride 1 unpadded, Cin a multiple of 64); shortcut: 1x1, stride s in both directions, unpadded,
// K2 input channels (a multiple of 64) on an H2 x W2 grid whose strided samples are a's output pixels
bool pair_applies(const ConvArgs &a, int dt, int H2, int W2, int K2, int Kp2, int stride) {
    return dt == SOL_BF16 && a.R == 1 && a.S == 1 && a.sh == 1 && a.sw == 1 && a.ph == 0 && a.pw == 0 && a.C % 64 == 0 && a.Kp == a.C &&
           K2 % 64 == 0 && Kp2 == K2 && stride >= 1 && (a.Ho - 1) * stride < H2 && (a.Wo - 1) * stride < W2 && a.pool == 0 &&
           a.Cout % 8 == 0 && (double)a.P * a.ldy < 4294967296.0 && (double)a.P * a.C * 2 < 2147483648.0 &&
           (double)a.N * H2 * W2 * K2 * 2 < 2147483648.0 && (double)a.Cout * (a.Kp > Kp2 ? a.Kp : Kp2) * 2 < 2147483648.0;
}

sol_status launch_conv_pair(ConvArgs a, const void *x2, const void *w2, const float *scale2, const float *shift2, int H2, int W2, int K2,
                            int Kp2, int stride, hipStream_t st) {
    if (a.P <= 0) return SOL_OK;
    if (a.C == 64 && K2 == 64 && stride == 1 && H2 == a.Ho && W2 == a.Wo) return launch_conv_pair_k64(a, x2, w2, scale2, shift2, st);
    a.res = nullptr;
    a.ntc = ceil_div(a.Cout, PR_BC);
    a.ntiles = ceil_div(a.P, PR_BP) * a.ntc;
    const int grid = ((a.ntiles + 7) / 8) * 8;
    const PairGeom g{x2, w2, scale2, shift2, H2, W2, K2, Kp2, stride};
    hipLaunchKernelGGL(conv_pair_kernel, dim3(grid), dim3(256), 0, st, a, g);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

sol_status launch_conv_pair_k64(ConvArgs a, const void *x2, const void *w2, const float *scale2, const float *shift2, hipStream_t st) {
    if (a.P <= 0) return SOL_OK;
    a.res = nullptr;
    a.ntc = ceil_div(a.Cout, PR_BC);
    a.ntiles = ceil_div(a.P, PR_BP) * a.ntc;
    const int grid = ((a.ntiles + 7) / 8) * 8;
    hipLaunchKernelGGL(conv_pair_k64_kernel, dim3(grid), dim3(256), 0, st, a, x2, w2, scale2, shift2);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

}  // namespace sol

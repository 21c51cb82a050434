// Shared host/device helpers of the HIP library (internal).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "../../include/sol.h"

namespace sol {

// ---- error reporting ---------------------------------------------------------------------------
void set_error(const char *fmt, ...);   // stores the text returned by sol_last_error()

#define SOL_FAIL(code, ...)            \
    do {                               \
        ::sol::set_error(__VA_ARGS__); \
        return (code);                 \
    } while (0)

#define SOL_REQUIRE(cond, code, ...) \
    do {                             \
        if (!(cond)) SOL_FAIL(code, __VA_ARGS__); \
    } while (0)

#define SOL_HIP(call)                                                                       \
    do {                                                                                    \
        hipError_t e_ = (call);                                                             \
        if (e_ != hipSuccess) SOL_FAIL(SOL_ERR_HIP, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

static inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline size_t dtype_size(int dt) { return dt == SOL_BF16 ? 2 : 4; }
static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
static inline size_t round_up(size_t a, size_t b) { return (a + b - 1) / b * b; }
static inline int out_size(int in, int k, int s, int p) { return (in + 2 * p - k) / s + 1; }

// reduction length of a packed convolution weight row (zero padded to one LDS row of 128 bytes)
static inline int packed_k(const sol_conv_desc &cd, int dt) {
    const int bk = dt == SOL_BF16 ? 64 : 32;
    return (int)round_up((size_t)cd.kh * cd.kw * cd.cin, bk);
}

// ---- device helpers ----------------------------------------------------------------------------
typedef uint16_t bf16_t;   // raw bf16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// two fp32 -> packed bf16 pair (low half = lo), round to nearest, ties to even: one v_cvt_pk_bf16_f32
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.f) & 0xffffu); }

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float *p) { return *p; }
    static __device__ __forceinline__ void store(float *p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t *p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(bf16_t *p, float v) { *p = f32_to_bf16(v); }
};

// ---- internal launchers (implemented in the .hip files) ------------------------------------------
// Division of a 32-bit unsigned by a run-time constant (multiply-high and shifts instead of the
// ~40-instruction software division; the divisor's magic number is computed on the host).
struct FastDiv {
    uint32_t d, mul, s1, s2;
    __host__ __device__ FastDiv() : d(1), mul(1), s1(0), s2(0) {}
    explicit FastDiv(uint32_t div) : d(div) {
        uint32_t l = 0;
        while ((1ull << l) < div) l++;
        mul = (uint32_t)(((1ull << 32) * ((1ull << l) - div)) / div + 1);
        s1 = l < 1 ? l : 1;
        s2 = l > 0 ? l - 1 : 0;
    }
#if defined(__HIPCC__)
    __device__ __forceinline__ uint32_t div(uint32_t n) const {
        const uint32_t t = __umulhi(mul, n);
        return (t + ((n - t) >> s1)) >> s2;
    }
    __device__ __forceinline__ void divmod(uint32_t n, uint32_t &q, uint32_t &r) const { q = div(n); r = n - q * d; }
#endif
};

struct ConvArgs {
    const void *x, *w;
    const float *scale, *shift;
    const void *res;
    void *y;
    int32_t *argmax;
    void *prepool;
    int N, H, W, C;          // input
    int Cout, R, S, sh, sw, ph, pw;
    int Ho, Wo;              // convolution output extent
    int Hy, Wy;              // stored output extent (pooled when pool != 0)
    int ldy;                 // elements between consecutive output pixels in y: Cout, or more when y is a channel slice of a
                             // wider tensor (a concatenation written in place); pool == 0 only
    int P;                   // GEMM rows: N*Ho*Wo, or N*Hy*Wy*4 with a fused 2x2 pool
    int Kp;                  // padded reduction length of a packed weight row
    int Ktot;                // R*S*C
    int act, pool;           // pool: 0 none, 1 max 2x2/2, 2 avg 2x2/2 (in the epilogue of any kernel), 3 max 3x3/2 pad 1 (stem-pool kernel only)
    const float *pre_scale, *pre_shift;   // not NULL: relu(pre_scale[c] * x + pre_shift[c]) is applied to every in-range input element before
                             // the contraction (BN + ReLU on the input side; taps in the padding stay 0); conv_igemm kernel only
    int ldx;                 // elements between consecutive input pixels in x: C, or more when x is a channel prefix of a wider tensor
    int Cvalid;              // input channels >= Cvalid read as 0 whatever the memory holds (C rounded up over a channel prefix); C when unused
    int ntc;                 // number of channel tiles (set by the launcher)
    int ntiles;
    int cpx;                 // > 0: each XCD owns cpx channel tiles (all pixel tiles); 0: a contiguous run of tiles
    FastDiv dw, dh;          // by Wo, Ho (by Wy, Hy with a fused pool): GEMM row -> pixel
};

struct PoolArgs {
    const void *x;
    void *y;
    int32_t *argmax;
    int N, H, W, C, Ho, Wo;
    int kh, kw, sh, sw, ph, pw;
    int kind, count_pad;
};

struct DwArgs {              // depthwise convolution: one filter per channel, weights [kh*kw][C]
    const void *x, *w, *res;
    const float *scale, *shift;
    void *y;
    int N, H, W, C, Ho, Wo;
    int kh, kw, sh, sw, ph, pw;
    int act;
};

// Convolution tile ids (pixels x channels per workgroup); also accepted as a debugging override.
// T_*: register-staged kernel (conv_igemm.hip).  D_*: LDS-DMA ring kernel (conv_dma.hip), suffix =
// row bytes per stage x ring stages.
enum {
    T_AUTO = 0, T_256x128 = 1, T_128x128 = 2, T_128x64 = 3, T_256x64 = 4, T_64x64 = 5, T_128x32 = 6, T_128x256 = 7,
    T_64x128 = 8,
    D_128x128_64x4 = 11, D_128x128_64x3 = 12, D_256x128_64x3 = 13, D_128x64_64x4 = 14, D_64x64_64x4 = 15,
    D_128x256_64x3 = 16, D_256x64_64x3 = 17, D_64x128_64x4 = 18,
    D_128x128_128x2 = 21, D_128x128_128x3 = 22, D_128x64_128x3 = 23, D_64x64_128x3 = 24,
    D_128x128_64x5 = 25, D_64x64_128x4 = 26, D_256x128_128x3 = 27, D_256x128_64x4 = 31, D_128x256_64x4 = 32, D_64x64_64x8 = 33,
    // H_*: 3x3 halo-in-LDS kernel (conv_halo.hip), suffix = patch DMA instructions per wave (s: single input chunk)
    H_256x128_x5 = 41, H_128x128_x3 = 42, H_256x64_x5 = 43, H_256x64_x6s = 44, H_256x64_x6s2 = 45, H_128x128_k2 = 46, H_64x128_k4 = 47, H_128x64_k4 = 48, H_64x64_k4 = 49, H_256x64_x6 = 50, H_FIRST = 41, H_LAST = 59,
    // G_*: eight-wave 1x1 GEMM kernel (conv_gemm8.hip); kN: reduction split N ways inside the workgroup, r64: 64-byte rows
    G_128x128_k2 = 61, G_256x128 = 62, G_128x256 = 63, G_64x128_k4 = 64, G_128x64_k4 = 65, G_256x256_r64 = 66, G_256x128_r64 = 67,
    G_64x64_k4 = 68, G_64x64_k4_deep = 69, G_64x32_k4_r256 = 70, G_FIRST = 61, G_LAST = 79,
    T_NO_HALO = 99   // automatic choice among the implicit-GEMM kernels only
};
int dma_tile_row_bytes(int tile);
sol_status launch_conv_dma(const ConvArgs &a, int dt, int tile, hipStream_t st);
bool gemm8_kernel_applies(const ConvArgs &a, int dt);
sol_status launch_conv_gemm8(const ConvArgs &a, int tile, hipStream_t st);
bool halo_kernel_applies(const ConvArgs &a, int dt);
int halo_choose_tile(const ConvArgs &a);
sol_status launch_conv_halo(const ConvArgs &a, int tile, hipStream_t st);
bool stem_kernel_applies(const ConvArgs &a, int dt);
sol_status launch_conv_stem(const ConvArgs &a, hipStream_t st);
// projection shortcut (1x1, stride s, K2 channels on an H2 x W2 grid) + the 1x1 convolution it is added to, in one kernel (conv_pair.hip)
bool pair_applies(const ConvArgs &a, int dt, int H2, int W2, int K2, int Kp2, int stride);
sol_status launch_conv_pair(ConvArgs a, const void *x2, const void *w2, const float *scale2, const float *shift2, int H2, int W2, int K2,
                            int Kp2, int stride, hipStream_t st);
bool stem_pool_applies(const ConvArgs &a, int dt, const sol_pool_desc &p);   // stem + ReLU + 3x3/2 max pool in one kernel
sol_status launch_conv_stem_pool(const ConvArgs &a, hipStream_t st);
// a whole stride-1 bottleneck (1x1 reduce, 3x3, 1x1 expand + identity shortcut, folded BN and ReLU each) in one kernel (conv_block.hip)
struct BlockLaunch {
    const void *x; void *y;                          // block input / output, NHWC [N][H][W][C4]
    const void *w1, *w2, *w3;                        // packed weights of the three convolutions
    const float *s1, *h1, *s2, *h2, *s3, *h3;        // their folded scale / shift
    int N, H, W, C4, WM;                             // WM: mid channels
};
bool block_kernel_applies(int dt, int N, int H, int W, int C4, int WM);
sol_status launch_conv_block(const BlockLaunch &b, hipStream_t st);
struct XrLaunch {
    const void *t, *r; void *y, *z;                  // expand input [P][WM], its shortcut [P][C4]; outputs y [P][C4], z [P][WZ]
    const void *w3, *w1;                             // packed weights [C4][WM], [WZ][C4]
    const float *s3, *h3, *s1, *h1;                  // folded scale / shift of the two layers
    long P; int WM, C4, WZ;
};
bool xr_kernel_applies(int dt, long P, int WM, int C4, int WZ);
sol_status launch_conv_xr(const XrLaunch &b, hipStream_t st);
bool linear_kernel_applies(const ConvArgs &a, int dt);
sol_status launch_linear(const ConvArgs &a, int dt, hipStream_t st);
sol_status launch_conv(const ConvArgs &a, int dt, int tile_override, hipStream_t st);
sol_status launch_pool(const PoolArgs &a, int dt, hipStream_t st);
sol_status launch_dwconv(const DwArgs &a, int dt, hipStream_t st);
sol_status launch_pack_dw(int C, int taps, int dt, const float *w, void *packed, hipStream_t st);
sol_status launch_gap(const void *x, void *y, int N, int HW, int C, int dt, hipStream_t st);
// copies a dense [rows][c] tensor into channels off .. off + c - 1 of a [rows][ldy] tensor (one part of a concatenation)
sol_status launch_concat_copy(const void *x, void *y, long rows, int c, int ldy, int off, int dt, hipStream_t st);
// cout_real / cin_real > 0: w holds that many filters / input channels, the rest of cd's are zero padding (pack only)
sol_status launch_pack(const sol_conv_desc &cd, int dt, const float *w, void *packed, bool unpack, hipStream_t st, int cout_real = 0,
                       int cin_real = 0);
sol_status launch_fold(int c, const float *gamma, const float *beta, const float *mean, const float *var,
                       const float *bias, float eps, float *scale, float *shift, hipStream_t st);

// training step (train.hip); `part` is scratch for the two-stage reductions
int col_reduce_chunks(int rows, int *rows_per_chunk);
sol_status launch_bn_stats(const void *z, int rows, int C, int dt, float eps, float *mean, float *var, float *invstd,
                           float *part, hipStream_t st);
sol_status launch_bn_apply(const void *z, const void *res, void *y, const float *mean, const float *invstd,
                           const float *gamma, const float *beta, long total, int C, int relu, int dt, hipStream_t st);
sol_status launch_grad_col_sums(const void *z, const void *dy, const void *y, const float *mean, const float *invstd,
                                int rows, int C, int relu, int dt, float *out0, float *out1, float *part, hipStream_t st);
sol_status launch_act_bn_bwd(const void *z, const void *dy, const void *y, const float *mean, const float *invstd,
                             const float *gamma, const float *dbeta, const float *dgamma, void *dz, void *dres,
                             int res_first, long total, int C, int relu, int bn, int rows, int dt, hipStream_t st);
sol_status launch_dilate(const void *dz, void *out, int N, int Ho, int Wo, int K, int Hd, int Wd, int sh, int sw, int dt,
                         hipStream_t st);
sol_status launch_pool_bwd(const PoolArgs &a, const void *dy, void *dx, int first, int dt, hipStream_t st);
sol_status launch_gap_bwd(const void *dy, void *dx, int N, int HW, int C, int first, int dt, hipStream_t st);
sol_status launch_softmax_ce(const void *logits, const int32_t *labels, void *dlogits, float *row_loss, float *loss, int N,
                             int C, int dt, hipStream_t st);

// Batched parameter update: up to SGD_MAX_SEG tensors updated, and up to PACK_MAX_SEG packed weight buffers rebuilt,
// by one launch each (a ResNet-18-shaped step otherwise spends ~100 launches on them).  The segment tables travel
// in the kernel arguments, so nothing is allocated or copied.
constexpr int SGD_MAX_SEG = 96, PACK_MAX_SEG = 64;
struct SgdBatch {
    int nseg;
    int first_block[SGD_MAX_SEG + 1];     // blocks [first_block[i], first_block[i+1]) work on segment i
    float *w[SGD_MAX_SEG], *v[SGD_MAX_SEG];
    const float *g[SGD_MAX_SEG];
    long n[SGD_MAX_SEG];
};
struct PackBatch {
    int nseg;
    int first_block[PACK_MAX_SEG + 1];
    const float *w[PACK_MAX_SEG];          // fp32 master, framework layout [K][C][R][S]
    void *out[PACK_MAX_SEG];
    int K[PACK_MAX_SEG], C[PACK_MAX_SEG], R[PACK_MAX_SEG], S[PACK_MAX_SEG], Kp[PACK_MAX_SEG], flip[PACK_MAX_SEG];
    int mode[PACK_MAX_SEG];                // how the segment's blocks are cut, set by pack_segment_blocks
};
// number of workgroups a segment takes in pack_batch_kernel (and the block-cutting mode, written to *mode)
int pack_segment_blocks(int K, int C, int R, int S, int Kp, int flip, int *mode);
constexpr int SGD_ELEMS_PER_BLOCK = 256 * 8, PACK_ELEMS_PER_BLOCK = 256 * 8;
sol_status launch_sgd_batch(const SgdBatch &b, float lr, float mu, hipStream_t st);
sol_status launch_pack_batch(const PackBatch &b, int dt, hipStream_t st);
sol_status launch_pack_flip(const sol_conv_desc &cd, int dt, const float *w, void *packed, hipStream_t st);
void wgrad_plan(const sol_tensor_desc &xd, const sol_conv_desc &cd, int Ho, int Wo, int *nsplit, size_t *part_floats);
// deferred_nsplit != NULL: only the first stage runs (split partials into `part`) and the number of splits is
// returned; the caller adds the partials of many layers in one launch_wgrad_reduce_batch
sol_status launch_wgrad(const sol_tensor_desc &xd, const void *x, const sol_conv_desc &cd, const void *dz, int Ho, int Wo,
                        float *dw, float *part, hipStream_t st, int *deferred_nsplit = nullptr);
// Second stage of the weight gradients of up to WRED_MAX_SEG layers in one launch: one workgroup per output channel
// of a layer adds that channel's split partials in split order and writes dW in framework layout.
constexpr int WRED_MAX_SEG = 64, WRED_MAX_PLANE = 12288;   // floats of one output channel's [taps][cin] plane held in LDS
struct WgradReduceBatch {
    int nseg;
    int first_block[WRED_MAX_SEG + 1];
    const float *part[WRED_MAX_SEG];
    float *dw[WRED_MAX_SEG];
    int nsplit[WRED_MAX_SEG], K[WRED_MAX_SEG], C[WRED_MAX_SEG], RS[WRED_MAX_SEG];
};
sol_status launch_wgrad_reduce_batch(const WgradReduceBatch &b, hipStream_t st);

}  // namespace sol

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

// fp32 -> bf16, round to nearest, ties to even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

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
    int P;                   // GEMM rows: N*Ho*Wo, or N*Hy*Wy*4 with a fused 2x2 pool
    int Kp;                  // padded reduction length of a packed weight row
    int Ktot;                // R*S*C
    int act, pool;           // pool: 0 none, 1 max 2x2/2, 2 avg 2x2/2
    int ntc;                 // number of channel tiles (set by the launcher)
    int ntiles;
};

struct PoolArgs {
    const void *x;
    void *y;
    int32_t *argmax;
    int N, H, W, C, Ho, Wo;
    int kh, kw, sh, sw, ph, pw;
    int kind, count_pad;
};

sol_status launch_conv(const ConvArgs &a, int dt, int tile_override, hipStream_t st);
sol_status launch_pool(const PoolArgs &a, int dt, hipStream_t st);
sol_status launch_gap(const void *x, void *y, int N, int HW, int C, int dt, hipStream_t st);
sol_status launch_pack(const sol_conv_desc &cd, int dt, const float *w, void *packed, bool unpack, hipStream_t st);
sol_status launch_fold(int c, const float *gamma, const float *beta, const float *mean, const float *var,
                       const float *bias, float eps, float *scale, float *shift, hipStream_t st);

}  // namespace sol

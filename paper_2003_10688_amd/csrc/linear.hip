// Linear layer for small batches:  y[m][o] = act( scale[o] * sum_i x[m][i] w[o][i] + shift[o] + res[m][o] ).
//
// With a batch of a few dozen rows the GEMM has one or two pixel tiles, so the convolution kernels, which
// parallelise over output tiles, leave most of the chip idle and walk the whole reduction in one workgroup.
// Here a workgroup owns 32 rows x 32 output features and its eight waves split the reduction between them;
// MFMA fragments (16 bytes of consecutive reduction elements of one row) are loaded straight from global
// memory into registers, sixteen steps in flight per wave (the kernel is latency-bound: for 2048 inputs that is
// the whole reduction in one round trip) -- x is tiny and
// L2-resident -- and the eight partial accumulators are added through LDS in a fixed order behind one barrier.
#include "conv_common.h"

namespace sol {

template <typename T>
__global__ void __launch_bounds__(512) linear_kernel(const ConvArgs a) {
    constexpr int EPC = 16 / (int)sizeof(T);       // reduction elements per fragment
    constexpr int UN = 16, NWV = 8;                // k-steps in flight per wave; waves per workgroup
    __shared__ float red[NWV][32][33];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 31, lh = lane >> 5;
    const int n0 = blockIdx.x * 32, m0 = blockIdx.y * 32;
    const int M = a.P, K = a.C, N = a.Cout;
    const T *__restrict__ xg = static_cast<const T *>(a.x);
    const T *__restrict__ wg = static_cast<const T *>(a.w);

    const bool wok = n0 + lr < N, xok = m0 + lr < M;
    const T *wp = wg + (size_t)(wok ? n0 + lr : 0) * a.Kp;
    const T *xp = xg + (size_t)(xok ? m0 + lr : 0) * K;
    const uint4 zero = make_uint4(0, 0, 0, 0);

    f32x16_t acc;
#pragma unroll
    for (int e = 0; e < 16; e++) acc[e] = 0.f;

    const int nsteps = (K + 2 * EPC - 1) / (2 * EPC);   // one step = 2*EPC reduction elements (both lane halves); K % EPC == 0
    for (int s0 = wave * UN; s0 < nsteps; s0 += NWV * UN) {
        // Every lane loads every step, from a clamped address (the start of a valid row), and what it must not use is
        // replaced by zeros after the last load is issued: a load behind a condition, or a use of its value between
        // the loads, makes the compiler wait for it before it issues the next one.
        uint4 fa[UN], fb[UN];
        auto k_of = [&](int u) { return (s0 + u) * 2 * EPC + lh * EPC; };   // < K, or: past the end / ragged last step
#pragma unroll
        for (int u = 0; u < UN; u++) {
            const int k = k_of(u), kk = k < K ? k : 0;
            fa[u] = *reinterpret_cast<const uint4 *>(wp + kk);
            fb[u] = *reinterpret_cast<const uint4 *>(xp + kk);
        }
        __builtin_amdgcn_sched_barrier(0);             // all 2 * UN loads are in flight before the first value is needed
#pragma unroll
        for (int u = 0; u < UN; u++) {
            const bool ok = k_of(u) < K;
            Mma<T>::run(acc, (ok && wok) ? fa[u] : zero, (ok && xok) ? fb[u] : zero);
        }
    }

    // accumulator register e of lane l: feature 8*(e/4) + 4*(l/32) + e%4, row l%32.  Every wave parks its partial
    // block, then each of the first 256 threads adds the eight partials of 4 outputs in wave order.
#pragma unroll
    for (int e = 0; e < 16; e++) red[wave][lr][8 * (e / 4) + 4 * lh + e % 4] = acc[e];
    __syncthreads();

    if (tid >= 256) return;
    const int row = tid >> 3, f0 = (tid & 7) * 4;
    const int m = m0 + row;
    if (m >= M) return;
    T *__restrict__ yg = static_cast<T *>(a.y);
    const T *__restrict__ resg = static_cast<const T *>(a.res);
#pragma unroll
    for (int e = 0; e < 4; e++) {
        const int o = n0 + f0 + e;
        if (o >= N) break;
        float t = 0.f;
#pragma unroll
        for (int w = 0; w < NWV; w++) t += red[w][row][f0 + e];
        t = t * (a.scale ? a.scale[o] : 1.f) + (a.shift ? a.shift[o] : 0.f);
        if (resg) t += Elem<T>::load(resg + (size_t)m * N + o);
        if (a.act == SOL_ACT_RELU) t = __builtin_fmaxf(t, 0.f);
        Elem<T>::store(yg + (size_t)m * a.ldy + o, t);
    }
}

// unpadded 1x1 "convolution" over a [rows,1,1,C] tensor with few rows, rows a whole number of 16-byte fragments.  The
// kernel reads x as P dense rows: with padding a [n,1,1,C] input has more output pixels than input rows (the padding
// pixels hold act(shift + residual)), which the gather kernels handle.
bool linear_kernel_applies(const ConvArgs &a, int dt) {
    const int frag = 16 / (int)dtype_size(dt);     // a fragment is 16 bytes of one row: rows must be whole fragments
    return a.R == 1 && a.S == 1 && a.H == 1 && a.W == 1 && a.ph == 0 && a.pw == 0 && a.Ho == 1 && a.Wo == 1 && a.P == a.N &&
           a.pool == 0 && a.P <= 1024 && a.C % frag == 0;
}

sol_status launch_linear(const ConvArgs &a, int dt, hipStream_t st) {
    const dim3 grid(ceil_div(a.Cout, 32), ceil_div(a.P, 32));
    if (dt == SOL_BF16)
        hipLaunchKernelGGL(linear_kernel<bf16_t>, grid, dim3(512), 0, st, a);
    else
        hipLaunchKernelGGL(linear_kernel<float>, grid, dim3(512), 0, st, a);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

}  // namespace sol

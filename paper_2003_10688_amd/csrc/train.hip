// Kernels of the training step: batch-statistics BN (forward statistics, apply, backward), the
// softmax cross-entropy loss, the weight-gradient contraction, the data movement of the strided
// data-gradient, pooling backward, and the SGD update.  The data-gradient contraction itself runs
// on the forward convolution kernels with spatially flipped, transposed weights.
//
// Every reduction is split into fixed chunks whose partial results are summed in a fixed order by a
// second launch, so results do not depend on scheduling (no floating-point atomics anywhere).
#include <math.h>

#include <type_traits>
#include "conv_common.h"
#include "vec_io.h"

namespace sol {

// ---- per-channel reductions over a [rows][C] tensor ----------------------------------------------
// 256 threads = 64 channels x 4 row phases; a block reduces `rpc` rows and writes one partial pair.
//   MODE 0: s0 = sum a
//   MODE 1: s0 = sum (a - mean)^2
//   MODE 2: g = relu ? (y > 0 ? b : 0) : b ;  s0 = sum g ;  s1 = sum g * (a - mean) * invstd  (a may be NULL)
template <typename T, int MODE>
__global__ void __launch_bounds__(256) col_reduce_kernel(const T *__restrict__ a, const T *__restrict__ b,
                                                         const T *__restrict__ y, const float *__restrict__ mean,
                                                         const float *__restrict__ invstd, float *__restrict__ part,
                                                         int rows, int C, int rpc, int relu) {
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int c = blockIdx.y * 64 + tx;
    const int r0 = blockIdx.x * rpc, r1 = min(rows, r0 + rpc);
    float s0 = 0.f, s1 = 0.f;
    if (c < C) {
        const float m = (MODE >= 1 && mean) ? mean[c] : 0.f;
        const float is = (MODE == 2 && invstd) ? invstd[c] : 0.f;
        for (int r = r0 + ty; r < r1; r += 4) {
            const size_t i = (size_t)r * C + c;
            if (MODE == 0) {
                s0 += Elem<T>::load(a + i);
            } else if (MODE == 1) {
                const float d = Elem<T>::load(a + i) - m;
                s0 += d * d;
            } else {
                float g = Elem<T>::load(b + i);
                if (relu && !(Elem<T>::load(y + i) > 0.f)) g = 0.f;
                s0 += g;
                if (a) s1 += g * ((Elem<T>::load(a + i) - m) * is);
            }
        }
    }
    __shared__ float red[2][4][64];
    red[0][ty][tx] = s0;
    red[1][ty][tx] = s1;
    __syncthreads();
    if (ty == 0 && c < C) {
        s0 = ((red[0][0][tx] + red[0][1][tx]) + red[0][2][tx]) + red[0][3][tx];
        s1 = ((red[1][0][tx] + red[1][1][tx]) + red[1][2][tx]) + red[1][3][tx];
        part[((size_t)blockIdx.x * 2 + 0) * C + c] = s0;
        part[((size_t)blockIdx.x * 2 + 1) * C + c] = s1;
    }
}

// Same reductions with 16-byte accesses (C % V == 0): 256 threads = 64/V channel groups x 256*V/64 row phases, every
// thread keeps V running sums; the phases are then added in order through LDS.
template <typename T, int V, int MODE>
__global__ void __launch_bounds__(256) col_reduce_vec_kernel(const T *__restrict__ a, const T *__restrict__ b,
                                                             const T *__restrict__ y, const float *__restrict__ mean,
                                                             const float *__restrict__ invstd, float *__restrict__ part,
                                                             int rows, int C, int rpc, int relu) {
    constexpr int CG = 64 / V, PH = 256 / CG;
    const int cg = threadIdx.x % CG, ph = threadIdx.x / CG;
    const int c0 = blockIdx.y * 64 + cg * V;
    const int r0 = blockIdx.x * rpc, r1 = min(rows, r0 + rpc);
    float s0[V], s1[V], m[V], is[V];
#pragma unroll
    for (int e = 0; e < V; e++) { s0[e] = 0.f; s1[e] = 0.f; m[e] = 0.f; is[e] = 0.f; }
    const bool cok = c0 < C;
    if (cok) {
#pragma unroll
        for (int e = 0; e < V; e++) {
            if (MODE >= 1 && mean) m[e] = mean[c0 + e];
            if (MODE == 2 && invstd) is[e] = invstd[c0 + e];
        }
        // Which tensors a row needs is fixed for the launch, so the row loop is instantiated per combination with
        // unconditional loads: behind a run-time condition every load would be waited for on the spot.  Four rows'
        // loads are issued before the first is used; the sums still run in row order.
        auto rows_loop = [&](auto HAS_A, auto RELU) {
            constexpr bool ha = decltype(HAS_A)::value, rl = decltype(RELU)::value;
            auto fetch = [&](int r, float (&va)[V], float (&vb)[V], float (&vy)[V]) {
                const size_t i = (size_t)r * C + c0;
                if constexpr (ha) VecIO<T, V>::load(a + i, va);
                if constexpr (MODE == 2) {
                    VecIO<T, V>::load(b + i, vb);
                    if constexpr (rl) VecIO<T, V>::load(y + i, vy);
                }
            };
            auto add = [&](const float (&va)[V], const float (&vb)[V], const float (&vy)[V]) {
#pragma unroll
                for (int e = 0; e < V; e++) {
                    if constexpr (MODE == 0) {
                        s0[e] += va[e];
                    } else if constexpr (MODE == 1) {
                        const float d = va[e] - m[e];
                        s0[e] += d * d;
                    } else {
                        float g = vb[e];
                        if constexpr (rl) { if (!(vy[e] > 0.f)) g = 0.f; }
                        s0[e] += g;
                        if constexpr (ha) s1[e] += g * ((va[e] - m[e]) * is[e]);
                    }
                }
            };
            int r = r0 + ph;
            for (; r + 3 * PH < r1; r += 4 * PH) {
                float va[4][V], vb[4][V], vy[4][V];
#pragma unroll
                for (int u = 0; u < 4; u++) fetch(r + u * PH, va[u], vb[u], vy[u]);
#pragma unroll
                for (int u = 0; u < 4; u++) add(va[u], vb[u], vy[u]);
            }
            for (; r < r1; r += PH) {
                float va[V], vb[V], vy[V];
                fetch(r, va, vb, vy);
                add(va, vb, vy);
            }
        };
        using std::true_type;
        using std::false_type;
        if constexpr (MODE <= 1) {
            rows_loop(true_type{}, false_type{});
        } else if (a) {
            if (relu) rows_loop(true_type{}, true_type{}); else rows_loop(true_type{}, false_type{});
        } else {
            if (relu) rows_loop(false_type{}, true_type{}); else rows_loop(false_type{}, false_type{});
        }
    }
    __shared__ float red[2][PH][64 + 1];
#pragma unroll
    for (int e = 0; e < V; e++) { red[0][ph][cg * V + e] = s0[e]; red[1][ph][cg * V + e] = s1[e]; }
    __syncthreads();
    const int tx = threadIdx.x, c = blockIdx.y * 64 + tx;
    if (tx < 64 && c < C) {
        float t0 = 0.f, t1 = 0.f;
#pragma unroll
        for (int p = 0; p < PH; p++) { t0 += red[0][p][tx]; t1 += red[1][p][tx]; }
        part[((size_t)blockIdx.x * 2 + 0) * C + c] = t0;
        part[((size_t)blockIdx.x * 2 + 1) * C + c] = t1;
    }
}

// Batch statistics in one trip over z: every block reduces its chunk of rows twice -- first to the chunk's sum,
// then (the chunk is a few tens of KB and still in the caches) to the chunk's sum of squared deviations from its
// own mean -- and col_merge_stats_kernel combines the chunks with the pairwise-update formula
//   M2 = sum_k M2_k + n_k (mean_k - mean)^2,
// which is as well conditioned as the two-pass definition but needs neither a second trip over HBM nor the
// two extra launches of a mean pass followed by a variance pass.
// part[chunk][0][c] = chunk mean, part[chunk][1][c] = chunk M2.
template <typename T, int V>
__global__ void __launch_bounds__(256) col_stats_vec_kernel(const T *__restrict__ a, float *__restrict__ part, int rows, int C, int rpc) {
    constexpr int CG = 64 / V, PH = 256 / CG;
    const int cg = threadIdx.x % CG, ph = threadIdx.x / CG;
    const int c0 = blockIdx.y * 64 + cg * V;
    const int r0 = blockIdx.x * rpc, r1 = min(rows, r0 + rpc);
    const bool cok = c0 < C;
    __shared__ float red[PH][64 + 1];
    __shared__ float cmean[64];
    float s[V], m[V];
    auto reduce_rows = [&](bool second) {
#pragma unroll
        for (int e = 0; e < V; e++) s[e] = 0.f;
        if (cok) {
            auto one_row = [&](int r) {
                float va[V];
                VecIO<T, V>::load(a + (size_t)r * C + c0, va);
#pragma unroll
                for (int e = 0; e < V; e++) {
                    const float d = va[e] - m[e];          // m = 0 in the first pass
                    s[e] += second ? d * d : d;
                }
            };
            int r = r0 + ph;
            for (; r + PH < r1; r += 2 * PH) { one_row(r); one_row(r + PH); }
            if (r < r1) one_row(r);
        }
#pragma unroll
        for (int e = 0; e < V; e++) red[ph][cg * V + e] = s[e];
        __syncthreads();
    };
#pragma unroll
    for (int e = 0; e < V; e++) m[e] = 0.f;
    reduce_rows(false);
    const int tx = threadIdx.x, c = blockIdx.y * 64 + tx;
    float csum = 0.f;
    if (tx < 64) {
#pragma unroll
        for (int p = 0; p < PH; p++) csum += red[p][tx];
        cmean[tx] = csum / (float)(r1 - r0);
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < V; e++) m[e] = cmean[cg * V + e];
    reduce_rows(true);
    if (tx < 64 && c < C) {
        float m2 = 0.f;
#pragma unroll
        for (int p = 0; p < PH; p++) m2 += red[p][tx];
        part[((size_t)blockIdx.x * 2 + 0) * C + c] = cmean[tx];
        part[((size_t)blockIdx.x * 2 + 1) * C + c] = m2;
    }
}

// mean / biased variance / 1/sqrt(var + eps) from the chunk means and chunk M2 of col_stats_vec_kernel; chunk k holds
// min(rpc, rows - k*rpc) rows.  64 channels x 16 chunk phases: phase p folds chunks p, p+16, ... into a running
// (count, mean, M2) triple with the pairwise update (one pass over the partials, four chunks' loads in flight),
// then one thread per channel folds the 16 phases in order.  The order depends on nothing but nchunks.
struct RunStats {
    float n, mean, m2;
    __device__ __forceinline__ void fold(float nk, float meank, float m2k) {
        const float nn = n + nk, d = meank - mean, f = nk / nn;     // nn > 0: nk >= 1 for every real chunk
        mean += d * f;
        m2 += m2k + d * d * n * f;
        n = nn;
    }
};
__global__ void __launch_bounds__(1024) col_merge_stats_kernel(const float *__restrict__ part, int nchunks, int C, int rows, int rpc,
                                                               float eps, float *__restrict__ mean, float *__restrict__ var,
                                                               float *__restrict__ inv) {
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int c = blockIdx.x * 64 + tx;
    __shared__ float red[3][16][64];
    RunStats rs{0.f, 0.f, 0.f};
    if (c < C) {
        int k = ty;
        for (; k + 48 < nchunks; k += 64) {
            float mk[4], qk[4];
#pragma unroll
            for (int u = 0; u < 4; u++) {
                mk[u] = part[((size_t)(k + 16 * u) * 2 + 0) * C + c];
                qk[u] = part[((size_t)(k + 16 * u) * 2 + 1) * C + c];
            }
#pragma unroll
            for (int u = 0; u < 4; u++) rs.fold((float)min(rpc, rows - (k + 16 * u) * rpc), mk[u], qk[u]);
        }
        for (; k < nchunks; k += 16)
            rs.fold((float)min(rpc, rows - k * rpc), part[((size_t)k * 2 + 0) * C + c], part[((size_t)k * 2 + 1) * C + c]);
    }
    red[0][ty][tx] = rs.n; red[1][ty][tx] = rs.mean; red[2][ty][tx] = rs.m2;
    __syncthreads();
    if (ty != 0 || c >= C) return;
    RunStats t{0.f, 0.f, 0.f};
#pragma unroll
    for (int p = 0; p < 16; p++)
        if (red[0][p][tx] > 0.f) t.fold(red[0][p][tx], red[1][p][tx], red[2][p][tx]);
    const float v = t.m2 / (float)rows;
    mean[c] = t.mean;
    var[c] = v;
    inv[c] = 1.f / sqrtf(v + eps);
}

// out0[c] = scale * sum_chunks part[chunk][0][c]; out1 likewise; with eps >= 0 also
// inv[c] = 1 / sqrt(out0[c] + eps)   (out0 = biased variance then)
__global__ void __launch_bounds__(1024) col_finalize_kernel(const float *__restrict__ part, int nchunks, int C, float scale,
                                                            float *__restrict__ out0, float *__restrict__ out1, float eps,
                                                            float *__restrict__ inv) {
    // 64 channels x 16 chunk phases; phase p adds chunks p, p+16, ... (4 independent loads in flight), the phases
    // are then added in order: the summation order depends on nothing but nchunks
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int c = blockIdx.x * 64 + tx;
    float s0 = 0.f, s1 = 0.f;
    if (c < C) {
        int k = ty;
        for (; k + 48 < nchunks; k += 64) {
            float a0[4], a1[4];
#pragma unroll
            for (int u = 0; u < 4; u++) {
                a0[u] = part[((size_t)(k + 16 * u) * 2 + 0) * C + c];
                a1[u] = part[((size_t)(k + 16 * u) * 2 + 1) * C + c];
            }
#pragma unroll
            for (int u = 0; u < 4; u++) { s0 += a0[u]; s1 += a1[u]; }
        }
        for (; k < nchunks; k += 16) {
            s0 += part[((size_t)k * 2 + 0) * C + c];
            s1 += part[((size_t)k * 2 + 1) * C + c];
        }
    }
    __shared__ float red[2][16][64];
    red[0][ty][tx] = s0;
    red[1][ty][tx] = s1;
    __syncthreads();
    if (ty != 0 || c >= C) return;
    s0 = 0.f; s1 = 0.f;
#pragma unroll
    for (int p = 0; p < 16; p++) { s0 += red[0][p][tx]; s1 += red[1][p][tx]; }
    s0 *= scale; s1 *= scale;
    if (out0) out0[c] = s0;
    if (out1) out1[c] = s1;
    if (inv) inv[c] = 1.f / sqrtf(s0 + eps);
}

// ---- elementwise passes -----------------------------------------------------------------------------
// y = act( gamma (z - mean) invstd + beta + res )        (BN with batch statistics, training forward)
// FIXC: 256 * V is a multiple of C, so a thread's V channels are the same in every iteration of its grid-stride
// loop and the per-channel operands are fetched once (otherwise they cost four loads per element of data).
template <typename T, int V, bool FIXC>
__global__ void __launch_bounds__(256) bn_apply_kernel(const T *__restrict__ z, const T *__restrict__ res, T *__restrict__ y,
                                                       const float *__restrict__ mean, const float *__restrict__ invstd,
                                                       const float *__restrict__ gamma, const float *__restrict__ beta,
                                                       long nvec, int C, int relu) {
    float m[V], is[V], ga[V], be[V];
    if (FIXC) {
        const int c0 = (int)((threadIdx.x * V) % C);
#pragma unroll
        for (int e = 0; e < V; e++) { m[e] = mean[c0 + e]; is[e] = invstd[c0 + e]; ga[e] = gamma[c0 + e]; be[e] = beta[c0 + e]; }
    }
    for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < nvec; i += (long)gridDim.x * blockDim.x) {
        if (!FIXC) {
            const int c0 = (int)((i * V) % C);
#pragma unroll
            for (int e = 0; e < V; e++) { m[e] = mean[c0 + e]; is[e] = invstd[c0 + e]; ga[e] = gamma[c0 + e]; be[e] = beta[c0 + e]; }
        }
        float v[V], r[V];
        VecIO<T, V>::load(z + i * V, v);
        if (res) VecIO<T, V>::load(res + i * V, r);
#pragma unroll
        for (int e = 0; e < V; e++) {
            float f = (v[e] - m[e]) * is[e] * ga[e] + be[e];
            if (res) f += r[e];
            if (relu) f = fmaxf(f, 0.f);
            v[e] = f;
        }
        VecIO<T, V>::store(y + i * V, v);
    }
}

// Backward through act / residual / BN of one layer:
//   g  = relu ? (y > 0 ? dy : 0) : dy
//   dres (+)= g                                   (when the layer has a residual input)
//   dz = gamma invstd (g - dbeta / M - xhat dgamma / M),   xhat = (z - mean) invstd      (BN)
//   dz = g                                                                               (no BN)
template <typename T, int V, bool FIXC>
__global__ void __launch_bounds__(256) act_bn_bwd_kernel(const T *__restrict__ z, const T *__restrict__ dy,
                                                         const T *__restrict__ y, const float *__restrict__ mean,
                                                         const float *__restrict__ invstd, const float *__restrict__ gamma,
                                                         const float *__restrict__ dbeta, const float *__restrict__ dgamma,
                                                         T *__restrict__ dz, T *dres, int res_first, long nvec, int C,
                                                         int relu, int bn, float inv_m) {
    float m[V], is[V], ga[V], db[V], dg[V];          // per-channel operands (see bn_apply_kernel for FIXC)
    auto fetch = [&](int c0) {
#pragma unroll
        for (int e = 0; e < V; e++) {
            m[e] = mean[c0 + e]; is[e] = invstd[c0 + e]; ga[e] = gamma[c0 + e]; db[e] = dbeta[c0 + e]; dg[e] = dgamma[c0 + e];
        }
    };
    if (FIXC && bn) fetch((int)((threadIdx.x * V) % C));
    for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < nvec; i += (long)gridDim.x * blockDim.x) {
        if (!FIXC && bn) fetch((int)((i * V) % C));
        float g[V], t[V];
        VecIO<T, V>::load(dy + i * V, g);
        if (relu) {
            VecIO<T, V>::load(y + i * V, t);
#pragma unroll
            for (int e = 0; e < V; e++)
                if (!(t[e] > 0.f)) g[e] = 0.f;
        }
        if (dres) {
            if (res_first) {
                VecIO<T, V>::store(dres + i * V, g);
            } else {
                VecIO<T, V>::load(dres + i * V, t);
#pragma unroll
                for (int e = 0; e < V; e++) t[e] += g[e];
                VecIO<T, V>::store(dres + i * V, t);
            }
        }
        if (bn) {
            VecIO<T, V>::load(z + i * V, t);
#pragma unroll
            for (int e = 0; e < V; e++) {
                const float xh = (t[e] - m[e]) * is[e];
                g[e] = ga[e] * is[e] * (g[e] - db[e] * inv_m - xh * dg[e] * inv_m);
            }
        }
        VecIO<T, V>::store(dz + i * V, g);
    }
}

// Zero-insertion of dz for a strided convolution: out[n][h*sh][w*sw][k] = dz[n][h][w][k], zero elsewhere,
// on an [N][Hd][Wd][K] grid; the data-gradient is then a stride-1 convolution over `out`.
template <typename T, int V>
__global__ void __launch_bounds__(256) dilate_kernel(const T *__restrict__ dz, T *__restrict__ out, int N, int Ho, int Wo,
                                                     int K, int Hd, int Wd, int sh, int sw) {
    const int kv = K / V;
    const long total = (long)N * Hd * Wd * kv;
    for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
        const int k = (int)(i % kv);
        long t = i / kv;
        const int w = (int)(t % Wd); t /= Wd;
        const int h = (int)(t % Hd);
        const int n = (int)(t / Hd);
        float v[V];
#pragma unroll
        for (int e = 0; e < V; e++) v[e] = 0.f;
        if (h % sh == 0 && w % sw == 0 && h / sh < Ho && w / sw < Wo)
            VecIO<T, V>::load(dz + ((((long)n * Ho + h / sh) * Wo + w / sw) * K + (long)k * V), v);
        VecIO<T, V>::store(out + i * V, v);
    }
}

// Pooling backward in gather form: an input pixel sums the gradients of the (few) windows that contain
// it -- for max pooling those whose stored winner index names it -- in row-major window order.
template <typename T, int V>
__global__ void __launch_bounds__(256) pool_bwd_kernel(const PoolArgs a, const T *__restrict__ dy, T *dx, int first) {
    const int cg = a.C / V;
    const long total = (long)a.N * a.H * a.W * cg;
    for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
        int g, iw, ih, n;
        if (total < (1L << 31)) {           // the usual case: 32-bit divisions (a 64-bit division is a long instruction sequence)
            const unsigned u = (unsigned)i, t0 = u / (unsigned)cg, t1 = t0 / (unsigned)a.W;
            g = (int)(u - t0 * (unsigned)cg); iw = (int)(t0 - t1 * (unsigned)a.W);
            n = (int)(t1 / (unsigned)a.H); ih = (int)(t1 - (unsigned)n * (unsigned)a.H);
        } else {
            g = (int)(i % cg);
            long t = i / cg;
            iw = (int)(t % a.W); t /= a.W;
            ih = (int)(t % a.H);
            n = (int)(t / a.H);
        }
        const int th = ih + a.ph - a.kh + 1, tw = iw + a.pw - a.kw + 1;
        const int p_lo = th <= 0 ? 0 : (th + a.sh - 1) / a.sh, p_hi = min(a.Ho - 1, (ih + a.ph) / a.sh);
        const int q_lo = tw <= 0 ? 0 : (tw + a.sw - 1) / a.sw, q_hi = min(a.Wo - 1, (iw + a.pw) / a.sw);
        float sum[V];
#pragma unroll
        for (int e = 0; e < V; e++) sum[e] = 0.f;
        if (a.kind == SOL_POOL_MAX && V % 4 == 0 && p_hi - p_lo <= 1 && q_hi - q_lo <= 1) {
            // at most 2 x 2 windows hold this pixel (window <= 2 strides): all their loads are issued together, from
            // clamped (always valid) addresses, and the windows that do not exist are masked out afterwards
            float d[4][V];
            int win[4][V];
            bool on[4];
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const int p = p_lo + (u >> 1), q = q_lo + (u & 1);
                on[u] = p <= p_hi && q <= q_hi;
                const long o = (((long)n * a.Ho + min(p, a.Ho - 1)) * a.Wo + min(q, a.Wo - 1)) * a.C + (long)g * V;
                VecIO<T, V>::load(dy + o, d[u]);
#pragma unroll
                for (int e = 0; e < V; e += 4) {
                    const int4 w4 = *reinterpret_cast<const int4 *>(a.argmax + o + e);
                    win[u][e] = w4.x; win[u][e + 1] = w4.y; win[u][e + 2] = w4.z; win[u][e + 3] = w4.w;
                }
            }
#pragma unroll
            for (int u = 0; u < 4; u++)                    // row-major window order, as the loop below
#pragma unroll
                for (int e = 0; e < V; e++)
                    if (on[u] && win[u][e] == ih * a.W + iw) sum[e] += d[u][e];
        } else
        for (int p = p_lo; p <= p_hi; p++)
            for (int q = q_lo; q <= q_hi; q++) {
                const long o = (((long)n * a.Ho + p) * a.Wo + q) * a.C + (long)g * V;
                float d[V];
                VecIO<T, V>::load(dy + o, d);
                if (a.kind == SOL_POOL_MAX) {
                    int win[V];
                    if constexpr (V % 4 == 0) {     // o is a multiple of V: 16-byte loads of the winners
#pragma unroll
                        for (int e = 0; e < V; e += 4) {
                            const int4 w4 = *reinterpret_cast<const int4 *>(a.argmax + o + e);
                            win[e] = w4.x; win[e + 1] = w4.y; win[e + 2] = w4.z; win[e + 3] = w4.w;
                        }
                    } else {
#pragma unroll
                        for (int e = 0; e < V; e++) win[e] = a.argmax[o + e];
                    }
#pragma unroll
                    for (int e = 0; e < V; e++)
                        if (win[e] == ih * a.W + iw) sum[e] += d[e];
                } else {
                    int cnt = a.kh * a.kw;
                    if (!a.count_pad) {
                        const int h0 = max(p * a.sh - a.ph, 0), h1 = min(p * a.sh - a.ph + a.kh, a.H);
                        const int w0 = max(q * a.sw - a.pw, 0), w1 = min(q * a.sw - a.pw + a.kw, a.W);
                        cnt = (h1 - h0) * (w1 - w0);
                    }
                    const float inv = 1.f / (float)cnt;
#pragma unroll
                    for (int e = 0; e < V; e++) sum[e] += d[e] * inv;
                }
            }
        if (!first) {
            float old[V];
            VecIO<T, V>::load(dx + i * V, old);
#pragma unroll
            for (int e = 0; e < V; e++) sum[e] += old[e];
        }
        VecIO<T, V>::store(dx + i * V, sum);
    }
}

// dx[n][p][c] (+)= dy[n][c] / HW
template <typename T, int V>
__global__ void __launch_bounds__(256) gap_bwd_kernel(const T *__restrict__ dy, T *dx, int N, int HW, int C, int first) {
    const int cg = C / V;
    const long total = (long)N * HW * cg;
    const float inv = 1.f / (float)HW;
    for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
        const int g = (int)(i % cg);
        const int n = (int)(i / ((long)cg * HW));
        float d[V], old[V];
        VecIO<T, V>::load(dy + ((long)n * C + (long)g * V), d);
        if (!first) VecIO<T, V>::load(dx + i * V, old);
#pragma unroll
        for (int e = 0; e < V; e++) d[e] = first ? d[e] * inv : old[e] + d[e] * inv;
        VecIO<T, V>::store(dx + i * V, d);
    }
}

// ---- softmax cross-entropy ------------------------------------------------------------------------------
__device__ __forceinline__ float block_reduce(float v, float *sm, bool is_max) {
    const int tid = threadIdx.x;
    sm[tid] = v;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (tid < s) sm[tid] = is_max ? fmaxf(sm[tid], sm[tid + s]) : sm[tid] + sm[tid + s];
        __syncthreads();
    }
    const float r = sm[0];
    __syncthreads();
    return r;
}

// One block per sample: row loss = logsumexp(l) - l[label]; dlogits = (softmax(l) - onehot) / N.
// A label outside [0, C) makes that row's loss NaN.
template <typename T>
__global__ void __launch_bounds__(256) softmax_ce_kernel(const T *__restrict__ logits, const int32_t *__restrict__ labels,
                                                         T *__restrict__ dlogits, float *__restrict__ row_loss, int N, int C) {
    __shared__ float sm[256];
    const int n = blockIdx.x, tid = threadIdx.x;
    const T *l = logits + (long)n * C;
    float mx = -INFINITY;
    for (int c = tid; c < C; c += 256) mx = fmaxf(mx, Elem<T>::load(l + c));
    mx = block_reduce(mx, sm, true);
    float s = 0.f;
    for (int c = tid; c < C; c += 256) s += expf(Elem<T>::load(l + c) - mx);
    s = block_reduce(s, sm, false);
    const int lab = labels[n];
    const float inv_s = 1.f / s, inv_n = 1.f / (float)N;
    for (int c = tid; c < C; c += 256) {
        const float p = expf(Elem<T>::load(l + c) - mx) * inv_s;
        Elem<T>::store(dlogits + (long)n * C + c, (p - (c == lab ? 1.f : 0.f)) * inv_n);
    }
    if (tid == 0) row_loss[n] = (lab >= 0 && lab < C) ? logf(s) + mx - Elem<T>::load(l + lab) : NAN;
}

__global__ void loss_mean_kernel(const float *__restrict__ row_loss, int N, float *__restrict__ loss) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        float s = 0.f;
        for (int i = 0; i < N; i++) s += row_loss[i];
        *loss = s / (float)N;
    }
}

// ---- SGD with momentum: v <- mu v + g ; w <- w - lr v ---------------------------------------------------------
// All parameter tensors of a network in one launch: block -> segment by a scan of the (scalar) block table.
__global__ void __launch_bounds__(256) sgd_batch_kernel(const SgdBatch b, float lr, float mu) {
    int seg = 0;
    while (seg + 1 < b.nseg && (int)blockIdx.x >= b.first_block[seg + 1]) seg++;
    float *__restrict__ w = b.w[seg], *__restrict__ v = b.v[seg];
    const float *__restrict__ g = b.g[seg];
    const long n = b.n[seg];
    const long i0 = (long)((int)blockIdx.x - b.first_block[seg]) * SGD_ELEMS_PER_BLOCK;
#pragma unroll
    for (int u = 0; u < SGD_ELEMS_PER_BLOCK / 256; u++) {
        const long i = i0 + u * 256 + threadIdx.x;
        if (i < n) {
            const float vel = mu * v[i] + g[i];
            v[i] = vel;
            w[i] -= lr * vel;
        }
    }
}

// All packed weight buffers of a network (forward order and, for the data gradient, flipped / transposed) rebuilt
// from the fp32 masters in one launch; same element maps as pack_weights_kernel / pack_weights_flip_kernel.
// Both maps transpose the channel axis against the filter taps, so a segment is cut into blocks whose reads AND
// writes are contiguous runs, with the transposition done in LDS:
//   mode 1 (forward pack): one block per output channel k; its [C][taps] plane is one contiguous run of the
//          master and becomes the contiguous packed row [taps][C] (+ zero padding);
//   mode 2 (flipped pack, C % 8 == 0, K % 64 == 0): one block per 8 input channels x KT output channels; the master
//          is read in runs of 8 x taps floats (one per k), the packed rows are written in runs of KT elements;
//   mode 0: any other shape, one gathered element per thread.
constexpr int PACK_PLANE = 9216;                   // floats of LDS per block
template <typename T>
__global__ void __launch_bounds__(256) pack_batch_kernel(const PackBatch b) {
    __shared__ float tile[PACK_PLANE + 128];
    int seg = 0;
    while (seg + 1 < b.nseg && (int)blockIdx.x >= b.first_block[seg + 1]) seg++;
    const float *__restrict__ w = b.w[seg];
    T *__restrict__ out = static_cast<T *>(b.out[seg]);
    const int K = b.K[seg], C = b.C[seg], R = b.R[seg], S = b.S[seg], Kp = b.Kp[seg], flip = b.flip[seg], mode = b.mode[seg];
    const int blk = (int)blockIdx.x - b.first_block[seg], RS = R * S;
    if (mode == 1) {
        const int n = C * RS;
        const float *src = w + (size_t)blk * n;
        // eight loads in flight per thread (a plain copy loop waits for every load before it issues the next)
        for (int i0 = threadIdx.x; i0 < n; i0 += 256 * 8) {                        // i = c * RS + tap
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; u++) v[u] = src[min(i0 + u * 256, n - 1)];
#pragma unroll
            for (int u = 0; u < 8; u++)
                if (i0 + u * 256 < n) tile[i0 + u * 256] = v[u];
        }
        __syncthreads();
        T *dst = out + (size_t)blk * Kp;
        for (int j = threadIdx.x; j < Kp; j += 256) {                               // j = tap * C + c
            const int tap = j / C, c = j - tap * C;
            Elem<T>::store(dst + j, j < n ? tile[c * RS + tap] : 0.f);
        }
        return;
    }
    if (mode == 2) {
        const int KT = K % 128 == 0 ? 128 : 64, nkb = K / KT, run = 8 * RS, pitch = run + 1;
        const int cb = blk / nkb, kb = blk - cb * nkb, c0 = cb * 8, k0 = kb * KT;
        for (int i0 = threadIdx.x; i0 < KT * run; i0 += 256 * 8) {                // eight loads in flight per thread
            float v[8];
            int dst[8];
#pragma unroll
            for (int u = 0; u < 8; u++) {
                const int i = min(i0 + u * 256, KT * run - 1);
                const int kk = i / run, rem = i - kk * run;                         // rem = cc * RS + tap
                dst[u] = kk * pitch + rem;
                v[u] = w[((size_t)(k0 + kk) * C + c0) * RS + rem];
            }
#pragma unroll
            for (int u = 0; u < 8; u++)
                if (i0 + u * 256 < KT * run) tile[dst[u]] = v[u];
        }
        __syncthreads();
        for (int o = threadIdx.x; o < KT * run; o += 256) {
            const int kk = o % KT, t2 = o / KT, tap = t2 % RS, cc = t2 / RS;        // tap: position in the flipped filter
            Elem<T>::store(out + (size_t)(c0 + cc) * Kp + (size_t)tap * K + k0 + kk, tile[kk * pitch + cc * RS + (RS - 1 - tap)]);
        }
        return;
    }
    const long total = (long)(flip ? C : K) * Kp;
    const long i0 = (long)blk * PACK_ELEMS_PER_BLOCK;
#pragma unroll
    for (int u = 0; u < PACK_ELEMS_PER_BLOCK / 256; u++) {
        const long i = i0 + u * 256 + threadIdx.x;
        if (i >= total) break;
        const unsigned row = (unsigned)i / (unsigned)Kp, j = (unsigned)i % (unsigned)Kp;    // packed buffers hold < 2^31 elements
        float v = 0.f;
        if (!flip) {                               // out[k][(r*S+s)*C + c]
            if (j < R * S * C) {
                const int c = j % C, tap = j / C, s = tap % S, r = tap / S;
                v = w[(((long)row * C + c) * R + r) * S + s];
            }
        } else {                                   // out[c][((R-1-r)*S + (S-1-s))*K + k]
            if (j < R * S * K) {
                const int k = j % K, tap = j / K, s = S - 1 - tap % S, r = R - 1 - tap / S;
                v = w[(((long)k * C + row) * R + r) * S + s];
            }
        }
        Elem<T>::store(out + i, v);
    }
}

int pack_segment_blocks(int K, int C, int R, int S, int Kp, int flip, int *mode) {
    const int RS = R * S;
    if (!flip && (long)C * RS <= PACK_PLANE) { *mode = 1; return K; }
    if (flip && C % 8 == 0 && K % 64 == 0 && (K % 128 == 0 ? 128 : 64) * (8 * RS + 1) <= PACK_PLANE + 128 && Kp == RS * K) {
        *mode = 2;
        return (C / 8) * (K / (K % 128 == 0 ? 128 : 64));
    }
    *mode = 0;
    const long total = (long)(flip ? C : K) * Kp;
    return (int)((total + PACK_ELEMS_PER_BLOCK - 1) / PACK_ELEMS_PER_BLOCK);
}

// Weights for the data-gradient: framework layout w[k][c][r][s] -> packed rows [c][((R-1-r)*S + (S-1-s))*K + k],
// i.e. the packed weight of a convolution with K input and C output channels and the filter flipped.
template <typename T>
__global__ void pack_weights_flip_kernel(const float *__restrict__ w, T *__restrict__ out, int K, int C, int R, int S,
                                         int Kp) {
    const long total = (long)C * Kp;
    for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
        const int c = (int)(i / Kp), j = (int)(i % Kp);
        float v = 0.f;
        if (j < R * S * K) {
            const int k = j % K, tap = j / K, s = S - 1 - tap % S, r = R - 1 - tap / S;
            v = w[(((long)k * C + c) * R + r) * S + s];
        }
        Elem<T>::store(out + i, v);
    }
}

// ---- weight gradient -------------------------------------------------------------------------------------
// dW[k][r][s][c] = sum over output pixels of dz[pixel][k] * x[pixel shifted by tap (r,s)][c]: a GEMM whose
// reduction runs over pixels, the slow axis of both NHWC operands.  A workgroup owns a 64 x 64 (k, c) block
// of one tap and a contiguous range of pixel groups; MFMA fragments (16 bytes of consecutive pixels for one
// channel) are gathered element-wise straight from global memory -- 32 lanes read 32 adjacent channels of one
// pixel, so every load instruction touches two contiguous segments -- with out-of-range taps, channel tails
// and row tails turned into zeros by the buffer range check.  Pixels are enumerated in groups of GP along an
// output row (GP = elements per 16 bytes); each half-wave takes one group per step, so one step reduces
// 2*GP pixels.  The four waves interleave steps and their accumulators are summed through LDS at the end;
// the block then writes one fp32 partial [k][tap][c], and a second launch adds the partials in order.
struct WgradArgs {
    const void *x, *dz;
    float *part;
    int N, H, W, C, K, R, S, sh, sw, ph, pw, Ho, Wo;
    int G, ngroups, nsteps, steps_per_split, nsplit, nkt, nct;
    uint32_t x_bytes, dz_bytes;
    FastDiv dG, dHo;
};

template <typename T> struct BufElem;
template <> struct BufElem<bf16_t> {
    static __device__ __forceinline__ uint32_t load(__amdgpu_buffer_rsrc_t r, uint32_t off) {
        return (uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(r, (int)off, 0, 0);
    }
    static __device__ __forceinline__ uint4 pack(const uint32_t e[8]) {
        return make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
    }
};
template <> struct BufElem<float> {
    static __device__ __forceinline__ uint32_t load(__amdgpu_buffer_rsrc_t r, uint32_t off) {
        return (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, 0);
    }
    static __device__ __forceinline__ uint4 pack(const uint32_t e[4]) { return make_uint4(e[0], e[1], e[2], e[3]); }
};

template <typename T>
__global__ void __launch_bounds__(256) wgrad_kernel(const WgradArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int GP = 16 / sizeof(T), ES = sizeof(T);
    __shared__ float red[64][65];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 31, h = lane >> 5;
    int bid = blockIdx.x;
    const int kt = bid % a.nkt; bid /= a.nkt;
    const int ct = bid % a.nct; bid /= a.nct;
    const int tap = bid % (a.R * a.S);
    const int split = bid / (a.R * a.S);
    const int r = tap / a.S, s = tap % a.S;
    const int k0 = kt * 64, c0 = ct * 64;

    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.x), 0, (int)a.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t zr = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.dz), 0, (int)a.dz_bytes, 0x00020000);

    f32x16_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

    const bool kok[2] = {k0 + lr < a.K, k0 + 32 + lr < a.K};
    const bool cok[2] = {c0 + lr < a.C, c0 + 32 + lr < a.C};
    const int s_begin = split * a.steps_per_split;
    const int s_end = min(a.nsteps, s_begin + a.steps_per_split);
    for (int t = s_begin + wave; t < s_end; t += 4) {
        const uint32_t g = 2u * (uint32_t)t + (uint32_t)h;
        uint32_t row, gq, n, op;
        a.dG.divmod(g, row, gq);
        a.dHo.divmod(row, n, op);
        const int q0 = (int)gq * GP;
        const bool gok = g < (uint32_t)a.ngroups;
        const int ih = (int)op * a.sh + r - a.ph;
        const bool rok = gok && (unsigned)ih < (unsigned)a.H;
        const uint32_t zbase = ((row * (uint32_t)a.Wo + (uint32_t)q0) * (uint32_t)a.K + (uint32_t)(k0 + lr)) * ES;
        const int iw0 = q0 * a.sw + s - a.pw;
        const uint32_t xbase = (((n * (uint32_t)a.H + (uint32_t)ih) * (uint32_t)a.W + (uint32_t)iw0) * (uint32_t)a.C +
                                (uint32_t)(c0 + lr)) * ES;
        uint32_t ea[2][GP], eb[2][GP];
#pragma unroll
        for (int e = 0; e < GP; e++) {
            const bool qok = gok && q0 + e < a.Wo;
            const bool wok = rok && qok && (unsigned)(iw0 + e * a.sw) < (unsigned)a.W;
#pragma unroll
            for (int i = 0; i < 2; i++) {
                const uint32_t oz = (qok && kok[i]) ? zbase + (uint32_t)(e * a.K + i * 32) * ES : 0xffffffffu;
                const uint32_t ox = (wok && cok[i]) ? xbase + (uint32_t)(e * a.sw * a.C + i * 32) * ES : 0xffffffffu;
                ea[i][e] = BufElem<T>::load(zr, oz);
                eb[i][e] = BufElem<T>::load(xr, ox);
            }
        }
        uint4 fa[2], fb[2];
#pragma unroll
        for (int i = 0; i < 2; i++) { fa[i] = BufElem<T>::pack(ea[i]); fb[i] = BufElem<T>::pack(eb[i]); }
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
            for (int j = 0; j < 2; j++) Mma<T>::run(acc[i][j], fa[i], fb[j]);
    }

    // accumulator register j of lane l holds D[row 8*(j/4) + 4*(l/32) + j%4][column l%32]; the waves add their
    // blocks one after the other, so the sum order is fixed
    for (int w = 0; w < 4; w++) {
        if (wave == w) {
#pragma unroll
            for (int i = 0; i < 2; i++)
#pragma unroll
                for (int j = 0; j < 2; j++)
#pragma unroll
                    for (int e = 0; e < 16; e++) {
                        float &d = red[i * 32 + 8 * (e / 4) + 4 * h + e % 4][j * 32 + lr];
                        d = w == 0 ? acc[i][j][e] : d + acc[i][j][e];
                    }
        }
        __syncthreads();
    }
    const size_t kstride = (size_t)a.R * a.S * a.C;
    float *out = a.part + (size_t)split * a.K * kstride;
    for (int i = tid; i < 64 * 64; i += 256) {
        const int kk = i >> 6, cc = i & 63;
        if (k0 + kk < a.K && c0 + cc < a.C)
            out[(size_t)(k0 + kk) * kstride + (size_t)tap * a.C + c0 + cc] =
                red[kk][cc];
    }
#endif
}

// Eight 2-byte LDS reads down a column of 128-byte rows = one MFMA fragment (rows 2q, 2q+1 -> low, high half of
// register q).  Opaque to the compiler: the caller waits (lgkmcnt) and only then packs the fragment with
// column8_landed() (anything that touched the registers before the data has landed would see stale values).  Plain
// zero-extending reads plus a pack: half-register (d16) loads do not preserve the other half on parts with SRAM ECC.
struct Column8 { unsigned e[8]; };
__device__ __forceinline__ void read_column8(Column8 &f, unsigned addr) {
    asm volatile("ds_read_u16 %0, %8 offset:0\n\t"
                 "ds_read_u16 %1, %8 offset:128\n\t"
                 "ds_read_u16 %2, %8 offset:256\n\t"
                 "ds_read_u16 %3, %8 offset:384\n\t"
                 "ds_read_u16 %4, %8 offset:512\n\t"
                 "ds_read_u16 %5, %8 offset:640\n\t"
                 "ds_read_u16 %6, %8 offset:768\n\t"
                 "ds_read_u16 %7, %8 offset:896"
                 : "=&v"(f.e[0]), "=&v"(f.e[1]), "=&v"(f.e[2]), "=&v"(f.e[3]), "=&v"(f.e[4]), "=&v"(f.e[5]), "=&v"(f.e[6]), "=&v"(f.e[7])
                 : "v"(addr));
}
// the same for a column whose rows are 16 bytes apart (the widened stem patch)
__device__ __forceinline__ void read_column8_16(Column8 &f, unsigned addr) {
    asm volatile("ds_read_u16 %0, %8 offset:0\n\t"
                 "ds_read_u16 %1, %8 offset:16\n\t"
                 "ds_read_u16 %2, %8 offset:32\n\t"
                 "ds_read_u16 %3, %8 offset:48\n\t"
                 "ds_read_u16 %4, %8 offset:64\n\t"
                 "ds_read_u16 %5, %8 offset:80\n\t"
                 "ds_read_u16 %6, %8 offset:96\n\t"
                 "ds_read_u16 %7, %8 offset:112"
                 : "=&v"(f.e[0]), "=&v"(f.e[1]), "=&v"(f.e[2]), "=&v"(f.e[3]), "=&v"(f.e[4]), "=&v"(f.e[5]), "=&v"(f.e[6]), "=&v"(f.e[7])
                 : "v"(addr));
}
__device__ __forceinline__ uint4 column8_landed(Column8 &f) {
    asm volatile("" : "+v"(f.e[0]), "+v"(f.e[1]), "+v"(f.e[2]), "+v"(f.e[3]), "+v"(f.e[4]), "+v"(f.e[5]), "+v"(f.e[6]), "+v"(f.e[7]));
    return make_uint4(f.e[0] | (f.e[1] << 16), f.e[2] | (f.e[3] << 16), f.e[4] | (f.e[5] << 16), f.e[6] | (f.e[7] << 16));
}

// One MFMA fragment -- 8 consecutive rows (pixels) of one 2-byte column (channel) per lane -- with two transposing LDS
// reads (ds_read_b64_tr_b16).  Within a group of 16 lanes, lane s supplies the address of 8 bytes (4 columns of one
// row) and lane i receives, as element j, column i % 4 of the 8 bytes that lane 4 * j + i / 4 addressed (lane layout
// measured on the part).  So when lane s addresses row s / 4, columns 4 * (s % 4) .. + 3, lane i ends up with rows
// 0..3 of column i: four consecutive pixels of its channel, low half of a register first, as the MFMA wants them.
// `addr` is that address for rows 0..3; rows 4..7 are 512 bytes (four 128-byte rows) further on.  Opaque to the
// compiler like Column8: wait (lgkmcnt), then tr8_landed().
typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
struct Tr8 { u32x2_t lo, hi; };
__device__ __forceinline__ void read_tr8(Tr8 &f, unsigned addr) {
    asm volatile("ds_read_b64_tr_b16 %0, %2 offset:0\n\t"
                 "ds_read_b64_tr_b16 %1, %2 offset:512"
                 : "=&v"(f.lo), "=&v"(f.hi)
                 : "v"(addr));
}
__device__ __forceinline__ uint4 tr8_landed(Tr8 &f) {
    asm volatile("" : "+v"(f.lo), "+v"(f.hi));
    return make_uint4(f.lo.x, f.lo.y, f.hi.x, f.hi.y);
}

// The same contraction with both operands staged through LDS (bf16, K % 8 == 0 and C % 8 == 0).  A stage is 64
// consecutive output pixels: their dz rows (64 channels = 128 bytes each) and the tap-shifted x rows travel
// HBM/L2 -> LDS by DMA, 16 bytes per lane, fully coalesced; rows that do not exist (pixel range end, padding taps,
// channel tails) get an out-of-range buffer offset and arrive as zeros.  Each of the four waves then takes one
// 16-pixel k-step of the stage: an MFMA fragment is 8 consecutive pixels of one channel, fetched by two transposing
// LDS reads (read_tr8).  One such read has 32 lanes fetch 64 contiguous bytes of each of 4 consecutive rows; rows
// 2, 3, 6, 7, ... sit 64 bytes further along than rows 0, 1, 4, 5, ... -- slot ^ 4, applied on the global side of the
// DMA -- so that the four rows cover all 64 banks once.  Ring of NS stages, one barrier per stage; partial sums and
// the second-stage reduction as above.
template <int NS>
__global__ void __launch_bounds__(256) wgrad_lds_kernel(const WgradArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)
    using namespace lds_pipe;
    constexpr int STAGE = 16384, L = 4;            // 8 KB of dz rows + 8 KB of x rows; DMA instructions per wave and stage
    __shared__ __align__(1024) unsigned char lds[NS * STAGE];
    static_assert(NS * STAGE >= 64 * 65 * 4, "the cross-wave reduction reuses the ring");
    const int tid = threadIdx.x, lane = tid & 63, lr = lane & 31, h = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int bid = blockIdx.x;
    const int kt = bid % a.nkt; bid /= a.nkt;
    const int ct = bid % a.nct; bid /= a.nct;
    const int tap = bid % (a.R * a.S);
    const int split = bid / (a.R * a.S);
    const int r = tap / a.S, s = tap % a.S;
    const int k0 = kt * 64, c0 = ct * 64;

    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.x), 0, (int)a.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t zr = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.dz), 0, (int)a.dz_bytes, 0x00020000);

    const int s_begin = split * a.steps_per_split, s_end = min(a.nsteps, s_begin + a.steps_per_split);   // stages of 64 pixels
    const int P = a.N * a.Ho * a.Wo;

    // DMA lanes: segment = 8 rows x 8 slots of 16 bytes; wave w owns dz segments 2w, 2w+1 and x segments 2w, 2w+1
    const int lslot = lane & 7, lrow = lane >> 3;
    unsigned zbase[2];
    int xrow[2], xslot[2];
#pragma unroll
    for (int i = 0; i < 2; i++) {
        const int row = (wave * 2 + i) * 8 + lrow;
        const int gs = lslot ^ (((row >> 1) & 1) << 2);        // global slot that lands in this lane's LDS slot
        zbase[i] = k0 + gs * 8 < a.K ? (unsigned)(row * a.K + k0 + gs * 8) * 2u : 0x80000000u;
        xrow[i] = row;
        xslot[i] = c0 + gs * 8 < a.C ? (c0 + gs * 8) * 2 : -1;
    }
    auto issue = [&](int st, int buf) {
        unsigned char *lz = lds + buf * STAGE, *lx = lz + 8192;
        const bool live = st < s_end;
        const unsigned zstage = (unsigned)st * 64u * (unsigned)a.K * 2u;
#pragma unroll
        for (int i = 0; i < 2; i++) {
            const unsigned zo = live ? zbase[i] + zstage : 0xffffffffu;   // pixels >= P lie beyond the tensor: zeros
            __builtin_amdgcn_raw_ptr_buffer_load_lds(zr, (__attribute__((address_space(3))) void *)(lz + (wave * 2 + i) * 1024), 16, zo, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 2; i++) {
            const uint32_t p = (uint32_t)st * 64u + (uint32_t)xrow[i];
            uint32_t row, ow, n, oh;
            a.dG.divmod(p, row, ow);                           // dG: division by Wo
            a.dHo.divmod(row, n, oh);
            const int ih = (int)oh * a.sh + r - a.ph, iw = (int)ow * a.sw + s - a.pw;
            const bool ok = live && p < (uint32_t)P && xslot[i] >= 0 && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
            const unsigned xo = ok ? (unsigned)(((n * (uint32_t)a.H + (uint32_t)ih) * (uint32_t)a.W + (uint32_t)iw) * (uint32_t)a.C) * 2u + (unsigned)xslot[i]
                                   : 0xffffffffu;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, (__attribute__((address_space(3))) void *)(lx + (wave * 2 + i) * 1024), 16, xo, 0, 0, 0);
        }
    };

    f32x16_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

    // transposing-read address of this lane for channel block i: row 16*wave + 8*h + s/4 (s = lane % 16), the 8 bytes
    // of channels 32*i + 16*((lane/16)%2) + 4*(s%4) .. +3, slot ^ 4 in rows whose bit 1 is set
    unsigned fbase[2];
    {
        const int sl = lane & 15, frow = 16 * wave + 8 * h + (sl >> 2);
#pragma unroll
        for (int i = 0; i < 2; i++) {
            const int slot = (i * 4 + ((lane >> 4) & 1) * 2 + ((sl & 3) >> 1)) ^ (((frow >> 1) & 1) << 2);
            fbase[i] = (unsigned)(frow * 128 + (slot << 4) + (sl & 1) * 8);
        }
    }

#pragma unroll
    for (int q = 0; q < NS - 1; q++) issue(s_begin + q, q);
    int buf = 0;
    for (int st = s_begin; st < s_end; st++) {
        wait_vmcnt<(NS - 2) * L>();                            // this wave's share of stage st has landed
        __builtin_amdgcn_s_barrier();                          // ... everyone's; and nobody still reads stage st-1 (a bare
                                                               // barrier: __syncthreads would also wait for the DMA in flight)
        issue(st + NS - 1, buf == 0 ? NS - 1 : buf - 1);
        // Fragment reads as opaque instructions (the compiler would otherwise wait for ALL outstanding DMA before
        // any LDS read): pixel e of a pair goes to the low half of a register, pixel e+1 to the high half.
        const unsigned zb = lds_addr(lds) + (unsigned)(buf * STAGE), xb = zb + 8192u;
        Tr8 ca[2], cb[2];
#pragma unroll
        for (int i = 0; i < 2; i++) {
            read_tr8(ca[i], zb + fbase[i]);
            read_tr8(cb[i], xb + fbase[i]);
        }
        wait_lgkmcnt<0>();
        uint4 fa[2], fb[2];
#pragma unroll
        for (int i = 0; i < 2; i++) { fa[i] = tr8_landed(ca[i]); fb[i] = tr8_landed(cb[i]); }
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
            for (int j = 0; j < 2; j++) Mma<bf16_t>::run(acc[i][j], fa[i], fb[j]);
        buf = buf + 1 == NS ? 0 : buf + 1;
    }
    wait_vmcnt<0>();                                           // zero-fill DMAs of the tail
    __syncthreads();                                           // the ring is dead: it becomes the reduction buffer

    float(*red)[65] = reinterpret_cast<float(*)[65]>(lds);
    for (int w = 0; w < 4; w++) {
        if (wave == w) {
#pragma unroll
            for (int i = 0; i < 2; i++)
#pragma unroll
                for (int j = 0; j < 2; j++)
#pragma unroll
                    for (int e = 0; e < 16; e++) {
                        float &d = red[i * 32 + 8 * (e / 4) + 4 * h + e % 4][j * 32 + lr];
                        d = w == 0 ? acc[i][j][e] : d + acc[i][j][e];
                    }
        }
        __syncthreads();
    }
    const size_t kstride = (size_t)a.R * a.S * a.C;
    float *out = a.part + (size_t)split * a.K * kstride;
    for (int i = tid; i < 64 * 64; i += 256) {
        const int kk = i >> 6, cc = i & 63;
        if (k0 + kk < a.K && c0 + cc < a.C) out[(size_t)(k0 + kk) * kstride + (size_t)tap * a.C + c0 + cc] = red[kk][cc];
    }
#endif
}

// Weight gradient of the 7x7 / stride-2 / pad-3 convolution over a 3-channel input (the ResNet-shaped stem), bf16.
// With Cin = 3 the generic kernels fill 3 of 64 columns of their (k, c) block.  Here, as in the forward stem kernel,
// a workgroup stages the input patch of an 8 x 16 block of output pixels in LDS widened to 4 channels, so that for
// a fixed filter row r the 28 (s, c) taps of neighbouring output pixels are 16 bytes apart: the contraction becomes
// D_r[k][s*4+c] = sum over pixels of dz[pixel][k] * patch[pixel, r][s*4+c], one 32-wide MFMA column block per filter
// row, and an MFMA fragment (8 consecutive output pixels of a row) is eight 2-byte LDS reads 16 bytes apart.  The
// block's dz rows arrive by DMA (double buffered); wave w accumulates filter rows w and w+4.  Persistent
// workgroups walk the pixel blocks; each writes one fp32 partial [k][tap][c] that wgrad_reduce_kernel adds in order.
constexpr int WS_TH = 8, WS_TW = 16, WS_IH = 2 * WS_TH + 5, WS_IW = 2 * WS_TW + 6;
__global__ void __launch_bounds__(256) wgrad_stem_kernel(const WgradArgs a, int tiles_h, int tiles_w, int ntiles) {
#if defined(__HIP_DEVICE_COMPILE__)
    using namespace lds_pipe;
    __shared__ __align__(1024) unsigned char dzl[2][128 * 128];          // dz rows of the block, 64 channels each
    __shared__ __align__(16) bf16_t xl[WS_IH * WS_IW * 4];               // widened input patch
    const int tid = threadIdx.x, lane = tid & 63, lr = lane & 31, h = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bf16_t *__restrict__ xg = static_cast<const bf16_t *>(a.x);
    const __amdgpu_buffer_rsrc_t zr = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.dz), 0, (int)a.dz_bytes, 0x00020000);

    for (int i = tid; i < WS_IH * WS_IW * 4; i += 256) xl[i] = 0;        // incl. the never-written pad column
    __syncthreads();

    // input patch of a block: (2*TH+5) x (2*TW+5) pixels of 3 channels, NP pixels per thread, one block ahead
    constexpr int NPIX = WS_IH * (WS_IW - 1), NP = (NPIX + 255) / 256;
    uint2 pv[NP];
    auto load_patch = [&](int tile) {
        const int tw = tile % tiles_w, t2 = tile / tiles_w;
        const int th = t2 % tiles_h, n = t2 / tiles_h;
#pragma unroll
        for (int i = 0; i < NP; i++) {
            const int e = tid + i * 256;
            const int ih = e / (WS_IW - 1), iw = e % (WS_IW - 1);
            const int gh = 2 * th * WS_TH - 3 + ih, gw = 2 * tw * WS_TW - 3 + iw;
            pv[i] = make_uint2(0, 0);
            if (e < NPIX && (unsigned)gh < (unsigned)a.H && (unsigned)gw < (unsigned)a.W) {
                const bf16_t *p = xg + (((long)n * a.H + gh) * a.W + gw) * 3;
                pv[i].x = (uint32_t)p[0] | ((uint32_t)p[1] << 16);
                pv[i].y = (uint32_t)p[2];
            }
        }
    };
    auto store_patch = [&]() {
#pragma unroll
        for (int i = 0; i < NP; i++) {
            const int e = tid + i * 256;
            if (e < NPIX) {
                const int ih = e / (WS_IW - 1), iw = e % (WS_IW - 1);
                *reinterpret_cast<uint2 *>(&xl[(ih * WS_IW + iw) * 4]) = pv[i];
            }
        }
    };
    // dz rows of a block: row py*16+px <- dz[n][p0+py][q0+px][0..63]; 16 segments of 8 rows x 8 slots, 4 per wave
    const int lslot = lane & 7, lrow = lane >> 3;
    auto issue_dz = [&](int tile, int buf) {
        const int tw = tile % tiles_w, t2 = tile / tiles_w;
        const int th = t2 % tiles_h, n = t2 / tiles_h;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int row = (wave * 4 + i) * 8 + lrow;
            const int p = th * WS_TH + (row >> 4), q = tw * WS_TW + (row & 15);
            const int gs = lslot ^ (((row >> 3) & 1) << 2);
            const bool ok = tile < ntiles && p < a.Ho && q < a.Wo && gs * 8 < a.K;
            const unsigned off = ok ? (unsigned)((((n * a.Ho + p) * a.Wo + q) * a.K + gs * 8) * 2) : 0xffffffffu;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(zr, (__attribute__((address_space(3))) void *)(&dzl[buf][(wave * 4 + i) * 1024]), 16, off, 0, 0, 0);
        }
    };

    f32x16_t acc[2][2];                                                   // [filter row slot][k block]
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;
    const bool two_rows = wave + 4 < 7;                                   // waves 0..2 own filter rows w and w+4, wave 3 row 3

    // fragment bases: dz column lr of k block i, rows 8h.. of a 16-pixel row of the block; patch taps lr = s*4+c
    unsigned fz[2];
#pragma unroll
    for (int i = 0; i < 2; i++) fz[i] = (unsigned)((8 * h) * 128 + (((i * 4 + (lr >> 3)) ^ (h << 2)) << 4) + (lr & 7) * 2);
    const unsigned fxl = lds_addr(xl) + (unsigned)((2 * 8 * h) * 8 + lr * 2);   // pixel 8h of the row, tap column lr

    int buf = 0;
    if ((int)blockIdx.x < ntiles) { load_patch(blockIdx.x); issue_dz(blockIdx.x, 0); }
    for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        __builtin_amdgcn_s_barrier();                                     // the previous block's patch and dz rows are no longer read
        store_patch();
        issue_dz(tile + gridDim.x, buf ^ 1);                              // the next block's dz rows (zeros past the end)
        wait_vmcnt<4>();                                                  // this block's dz rows have landed (this wave's share)
        wait_lgkmcnt<0>();                                                // ... and its patch stores
        __builtin_amdgcn_s_barrier();                                     // bare barriers: the DMA just issued stays in flight
        if (tile + (int)gridDim.x < ntiles) load_patch(tile + gridDim.x); // in flight under the MFMAs
        const unsigned zb = lds_addr(&dzl[buf][0]);
#pragma unroll
        for (int py = 0; py < WS_TH; py++) {                              // one k-step = the 16 pixels of block row py
            Column8 ca[2], cb[2];
#pragma unroll
            for (int i = 0; i < 2; i++) read_column8(ca[i], zb + (unsigned)(py * 16 * 128) + fz[i]);
            read_column8_16(cb[0], fxl + (unsigned)(((2 * py + wave) * WS_IW) * 8));
            if (two_rows) read_column8_16(cb[1], fxl + (unsigned)(((2 * py + wave + 4) * WS_IW) * 8));
            wait_lgkmcnt<0>();
            uint4 fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; i++) fa[i] = column8_landed(ca[i]);
            fb[0] = column8_landed(cb[0]);
#pragma unroll
            for (int i = 0; i < 2; i++) Mma<bf16_t>::run(acc[0][i], fa[i], fb[0]);
            if (two_rows) {
                fb[1] = column8_landed(cb[1]);
#pragma unroll
                for (int i = 0; i < 2; i++) Mma<bf16_t>::run(acc[1][i], fa[i], fb[1]);
            }
        }
        buf ^= 1;
    }
    wait_vmcnt<0>();

    // partial of this workgroup: part[wg][k][tap = r*7+s][c]; accumulator register e of lane l holds
    // D[k = 8*(e/4) + 4*(l/32) + e%4 (+32 i)][column l%32 = s*4 + c]
    float *out = a.part + (size_t)blockIdx.x * a.K * 147;
    const int sx = lr >> 2, c = lr & 3;
#pragma unroll
    for (int slot = 0; slot < 2; slot++) {
        const int r = wave + 4 * slot;
        if (r < 7 && sx < 7 && c < 3) {
#pragma unroll
            for (int i = 0; i < 2; i++)
#pragma unroll
                for (int e = 0; e < 16; e++) {
                    const int k = i * 32 + 8 * (e / 4) + 4 * h + e % 4;
                    if (k < a.K) out[((size_t)k * 49 + r * 7 + sx) * 3 + c] = acc[slot][i][e];
                }
        }
    }
#endif
}

// ---- 3x3 / stride 1 / pad 1: one workgroup per filter ROW -------------------------------------------------------
// wgrad_lds_kernel gives every filter tap its own workgroups, so the dz tile of a stage is fetched nine times and
// the x tile once per tap: 16 KB through the DMA path per 16 MFMAs, which is what bounds it.  Here a workgroup owns
// the three taps of one filter row r.  A stage is nr = 64 / W whole output rows (nr * W <= 64 pixels): their dz rows
// and ONE run of x pixels -- output pixel m with tap s reads patch row m + s, the flattened-shift trick of the halo
// forward kernel (input pixel index = output pixel index + (r-1) W + (s-1)) -- serve 36 MFMAs per 17 KB.  Because a
// stage is whole image rows, a lane's pixels keep their column from stage to stage: taps that leave the image on
// the left / right are redirected, once and for all, to a patch row that the DMA always zero-fills, and rows whose
// input row oh + r - 1 lies outside the image have their dz row zero-filled by the DMA instead (x then holds a
// neighbouring image's finite values, times zero).  Nothing in the loop computes an address: LDS offsets are per-lane
// constants plus an immediate (the ring is unrolled), DMA offsets a per-lane constant plus a scalar.
// Wave w owns the 32 x 32 block (w % 2, w / 2) of the 64 x 64 tile for all three taps and all four 16-pixel k-steps
// of a stage, so there is no cross-wave sum at the end.
constexpr int WR_NS = 3, WR_XROWS = 96, WR_STAGE = 8192 + WR_XROWS * 128, WR_L = 5, WR_ZROW = WR_XROWS - 1;
template <int IMM> __device__ __forceinline__ void read_tr4(u32x2_t &d, unsigned addr) {
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=&v"(d) : "v"(addr), "n"(IMM));
}
__global__ void __launch_bounds__(256) wgrad_row_kernel(const WgradArgs a, int nr) {
#if defined(__HIP_DEVICE_COMPILE__)
    using namespace lds_pipe;
    static_assert(WR_NS * WR_STAGE + 1024 <= 65536, "LDS offsets are 16-bit immediates");
    __shared__ __align__(1024) unsigned char lds[WR_NS * WR_STAGE];
    const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, sl = lane & 15;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int bid = blockIdx.x;
    const int kt = bid % a.nkt; bid /= a.nkt;
    const int ct = bid % a.nct; bid /= a.nct;
    const int r = bid % a.R;
    const int split = bid / a.R;
    const int k0 = kt * 64, c0 = ct * 64, kc = wave & 1, cc = wave >> 1;
    const int W = a.W, H = a.H, G = a.N * H, npx = nr * W;

    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.x), 0, (int)a.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t zr = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.dz), 0, (int)a.dz_bytes, 0x00020000);
    const int s_begin = split * a.steps_per_split, s_end = min(a.nsteps, s_begin + a.steps_per_split);

    // ---- DMA lanes: a segment is 8 rows x 8 slots of 16 bytes.  Wave w owns dz segments 2w, 2w+1 and x segments
    // 2w, 2w+1, 8+w.  slot ^ 4 in rows whose bit 1 is set (bank spread of the transposing reads).
    const int lslot = lane & 7, lrow = lane >> 3;
    unsigned zoff[2], xoff[3];
    int zrow_g[2], zrow_oh[2];                     // global (n, oh) row index of this lane's dz row, and its oh
#pragma unroll
    for (int i = 0; i < 2; i++) {
        const int m = (wave * 2 + i) * 8 + lrow, gs = lslot ^ (((m >> 1) & 1) << 2);
        zoff[i] = (m < npx && k0 + gs * 8 < a.K) ? (unsigned)(m * a.K + k0 + gs * 8) * 2u : 0x80000000u;
        zrow_g[i] = s_begin * nr + m / W;
        zrow_oh[i] = zrow_g[i] % H;
    }
#pragma unroll
    for (int i = 0; i < 3; i++) {
        const int j = (i < 2 ? wave * 2 + i : 8 + wave) * 8 + lrow, gs = lslot ^ (((j >> 1) & 1) << 2);
        // patch row j of stage st = input pixel st * npx + (r - 1) W - 1 + j (negative: wraps out of range -> zeros)
        xoff[i] = (j < npx + 2 && c0 + gs * 8 < a.C) ? (unsigned)(((r - 1) * W - 1 + j) * a.C + c0 + gs * 8) * 2u : 0x80000000u;
    }
    const int nr_mod = nr % H;
    auto issue = [&](int st, int buf) {
        unsigned char *lz = lds + buf * WR_STAGE, *lx = lz + 8192;
        const bool live = st < s_end;
        const unsigned zstage = (unsigned)st * (unsigned)npx * (unsigned)a.K * 2u, xstage = (unsigned)st * (unsigned)npx * (unsigned)a.C * 2u;
#pragma unroll
        for (int i = 0; i < 2; i++) {
            const bool ok = live && zrow_g[i] < G && (unsigned)(zrow_oh[i] + r - 1) < (unsigned)H;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(zr, (__attribute__((address_space(3))) void *)(lz + (wave * 2 + i) * 1024), 16,
                                                     ok ? zoff[i] + zstage : 0xffffffffu, 0, 0, 0);
            zrow_g[i] += nr;                       // the next stage this lane issues is st + 1
            zrow_oh[i] += nr_mod;
            zrow_oh[i] -= zrow_oh[i] >= H ? H : 0;
        }
#pragma unroll
        for (int i = 0; i < 3; i++)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, (__attribute__((address_space(3))) void *)(lx + (i < 2 ? wave * 2 + i : 8 + wave) * 1024), 16,
                                                     live ? xoff[i] + xstage : 0xffffffffu, 0, 0, 0);
    };

    // ---- transposing-read addresses (per-lane constants, stage buffer 0): lane sl of a 16-lane group addresses
    // pixel row (sl >> 2) [+4 for the upper half] of its k-step, the 8 bytes of channels 4 (sl & 3) .. +3 of its block
    unsigned zaddr[4], xaddr[4][3][2];
    {
        const int slot_z = kc * 4 + ((lane >> 4) & 1) * 2 + ((sl & 3) >> 1), slot_x = cc * 4 + ((lane >> 4) & 1) * 2 + ((sl & 3) >> 1);
        const unsigned lo = (unsigned)(sl & 1) * 8u, base = lds_addr(lds);
#pragma unroll
        for (int ks = 0; ks < 4; ks++) {
            const int m0 = 16 * ks + 8 * h + (sl >> 2);
            zaddr[ks] = base + (unsigned)(m0 * 128 + ((slot_z ^ (((m0 >> 1) & 1) << 2)) << 4)) + lo;
#pragma unroll
            for (int e = 0; e < 2; e++) {
                const int m = m0 + 4 * e, ow = m % W;
#pragma unroll
                for (int t = 0; t < 3; t++) {
                    const bool ok = (unsigned)(ow + t - 1) < (unsigned)W;
                    const int j = ok ? m + t : WR_ZROW;
                    xaddr[ks][t][e] = base + 8192u + (unsigned)(j * 128 + ((slot_x ^ (((j >> 1) & 1) << 2)) << 4)) + lo;
                }
            }
        }
    }

    f32x16_t acc[3];
#pragma unroll
    for (int t = 0; t < 3; t++)
#pragma unroll
        for (int e = 0; e < 16; e++) acc[t][e] = 0.f;

    issue(s_begin, 0);
    issue(s_begin + 1, 1);
    auto stage = [&](auto BUF, int st) {
        constexpr int buf = decltype(BUF)::value, IMM = buf * WR_STAGE;
        wait_vmcnt<(WR_NS - 2) * WR_L>();                      // this wave's share of stage st has landed
        __builtin_amdgcn_s_barrier();                          // ... everyone's; and nobody still reads stage st-1
        issue(st + WR_NS - 1, (buf + WR_NS - 1) % WR_NS);
        // fragments of k-step ks+1 are requested before the MFMAs of k-step ks are issued
        Tr8 fz[2], fx[2][3];
        auto request = [&](auto KS) {
            constexpr int ks = decltype(KS)::value, set = ks & 1;
            read_tr4<IMM>(fz[set].lo, zaddr[ks]);
            read_tr4<IMM + 512>(fz[set].hi, zaddr[ks]);
#pragma unroll
            for (int t = 0; t < 3; t++) {
                read_tr4<IMM>(fx[set][t].lo, xaddr[ks][t][0]);
                read_tr4<IMM>(fx[set][t].hi, xaddr[ks][t][1]);
            }
        };
        request(std::integral_constant<int, 0>{});
        static_for<4>([&](auto KS) {
            constexpr int ks = decltype(KS)::value, set = ks & 1;
            if constexpr (ks + 1 < 4) {
                request(std::integral_constant<int, ks + 1>{});
                wait_lgkmcnt<8>();                             // only the eight reads just requested may be outstanding
            } else {
                wait_lgkmcnt<0>();
            }
            const uint4 fa = tr8_landed(fz[set]);
#pragma unroll
            for (int t = 0; t < 3; t++) Mma<bf16_t>::run(acc[t], fa, tr8_landed(fx[set][t]));
        });
    };
    // whole rounds of the ring; stages past s_end are zero-filled by the DMA and add nothing
    for (int st = s_begin; st < s_end; st += WR_NS) {
        stage(std::integral_constant<int, 0>{}, st);
        stage(std::integral_constant<int, 1>{}, st + 1);
        stage(std::integral_constant<int, 2>{}, st + 2);
    }
    wait_vmcnt<0>();                                           // zero-fill DMAs of the tail

    const size_t kstride = (size_t)a.R * a.S * a.C;
    float *out = a.part + (size_t)split * a.K * kstride;
    const int cw = c0 + cc * 32 + (lane & 31);
#pragma unroll
    for (int t = 0; t < 3; t++)
#pragma unroll
        for (int e = 0; e < 16; e++) {
            const int kk = k0 + kc * 32 + 8 * (e / 4) + 4 * h + e % 4;
            if (kk < a.K && cw < a.C) out[(size_t)kk * kstride + (size_t)(r * 3 + t) * a.C + cw] = acc[t][e];
        }
#endif
}

// dW[k][c][r][s] (framework layout) = sum over splits of part[split][k][r*S+s][c], added in split order
__global__ void __launch_bounds__(256) wgrad_reduce_kernel(const float *__restrict__ part, int nsplit, float *__restrict__ dw,
                                                           int K, int C, int RS) {
    const long total = (long)K * RS * C;
    for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
        float s = 0.f;
        for (int k = 0; k < nsplit; k++) s += part[(size_t)k * total + i];
        const int c = (int)(i % C);
        const long t = i / C;
        const int tap = (int)(t % RS), ko = (int)(t / RS);
        dw[((long)ko * C + c) * RS + tap] = s;
    }
}

// The same sum for many layers at once.  A workgroup (1024 threads) owns one output channel ko of one layer.  Its
// [taps][cin] plane has n floats in each of nsplit partials; small planes come with many splits (the 7x7 stem:
// 147 floats x 256 splits), so the threads form PH phases x U units (a unit = 4 floats when n % 4 == 0, else 1):
// phase p adds splits p, p+PH, ... (four loads in flight), the phases are added in order through LDS, and the plane
// is written transposed to [cin][taps] -- contiguous in dW -- so both sides of the transposition are coalesced.
// The order of every sum depends on the layer's shape only.
__global__ void __launch_bounds__(1024) wgrad_reduce_batch_kernel(const WgradReduceBatch b) {
    __shared__ __align__(16) float plane[WRED_MAX_PLANE];
    int seg = 0;
    while (seg + 1 < b.nseg && (int)blockIdx.x >= b.first_block[seg + 1]) seg++;
    const int ko = (int)blockIdx.x - b.first_block[seg];
    const int C = b.C[seg], RS = b.RS[seg], n = C * RS, nsplit = b.nsplit[seg];
    const size_t total = (size_t)b.K[seg] * n;
    const float *__restrict__ src = b.part[seg] + (size_t)ko * n;
    const bool vec = (n & 3) == 0;
    const int units = vec ? n >> 2 : n, upad = (units + 63) & ~63;
    const int PH = max(1, min(min(1024 / upad, WRED_MAX_PLANE / n), nsplit));
    const int ustride = upad * PH <= 1024 ? upad : 1024;     // PH == 1: all threads walk the units
    const int ph = PH > 1 ? (int)threadIdx.x / upad : 0;
    if (ph < PH) {
        for (int u = PH > 1 ? (int)threadIdx.x - ph * upad : (int)threadIdx.x; u < units; u += ustride) {
            if (vec) {
                float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
                int k = ph;
                for (; k + 3 * PH < nsplit; k += 4 * PH) {
                    float4 v[4];
#pragma unroll
                    for (int j = 0; j < 4; j++) v[j] = *reinterpret_cast<const float4 *>(src + (size_t)(k + j * PH) * total + 4 * u);
#pragma unroll
                    for (int j = 0; j < 4; j++) { s.x += v[j].x; s.y += v[j].y; s.z += v[j].z; s.w += v[j].w; }
                }
                for (; k < nsplit; k += PH) {
                    const float4 v = *reinterpret_cast<const float4 *>(src + (size_t)k * total + 4 * u);
                    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
                }
                *reinterpret_cast<float4 *>(plane + ph * n + 4 * u) = s;
            } else {
                float s = 0.f;
                int k = ph;
                for (; k + 3 * PH < nsplit; k += 4 * PH) {
                    float v[4];
#pragma unroll
                    for (int j = 0; j < 4; j++) v[j] = src[(size_t)(k + j * PH) * total + u];
                    s = (((s + v[0]) + v[1]) + v[2]) + v[3];
                }
                for (; k < nsplit; k += PH) s += src[(size_t)k * total + u];
                plane[ph * n + u] = s;
            }
        }
    }
    __syncthreads();
    float *__restrict__ dst = b.dw[seg] + (size_t)ko * n;
    for (int o = threadIdx.x; o < n; o += 1024) {      // o = c * RS + tap
        const int c = o / RS, tap = o - c * RS;
        float s = 0.f;
        for (int p = 0; p < PH; p++) s += plane[p * n + tap * C + c];
        dst[o] = s;
    }
}

sol_status launch_wgrad_reduce_batch(const WgradReduceBatch &b, hipStream_t st) {
    if (b.nseg <= 0 || b.first_block[b.nseg] <= 0) return SOL_OK;
    hipLaunchKernelGGL(wgrad_reduce_batch_kernel, dim3(b.first_block[b.nseg]), dim3(1024), 0, st, b);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

// ---- launchers ---------------------------------------------------------------------------------------------
static inline int grid_for(long n) { return (int)std::min<long>((n + 255) / 256, 8192); }

#define SOL_DISPATCH_TV(dt, C, STMT)                                       \
    do {                                                                   \
        if ((dt) == SOL_BF16) {                                            \
            typedef bf16_t T;                                              \
            if ((C) % 8 == 0) { constexpr int V = 8; STMT; } else { constexpr int V = 1; STMT; } \
        } else {                                                           \
            typedef float T;                                               \
            if ((C) % 4 == 0) { constexpr int V = 4; STMT; } else { constexpr int V = 1; STMT; } \
        }                                                                  \
    } while (0)

int col_reduce_chunks(int rows, int *rpc_out) {
    int rpc = std::max(64, ceil_div(rows, 512));
    rpc = (rpc + 3) / 4 * 4;
    if (rpc_out) *rpc_out = rpc;
    return std::max(1, ceil_div(rows, rpc));
}

// mean / biased variance / 1/sqrt(var+eps) over the rows of z [rows][C]; part: 2*C*chunks floats
sol_status launch_bn_stats(const void *z, int rows, int C, int dt, float eps, float *mean, float *var, float *invstd,
                           float *part, hipStream_t st) {
    int rpc;
    const int nch = col_reduce_chunks(rows, &rpc);
    const dim3 grid(nch, ceil_div(C, 64));
    const int fg = ceil_div(C, 64);
    if ((dt == SOL_BF16 && C % 8 == 0) || (dt != SOL_BF16 && C % 4 == 0)) {     // one trip over z, two launches
        if (dt == SOL_BF16)
            hipLaunchKernelGGL((col_stats_vec_kernel<bf16_t, 8>), grid, dim3(256), 0, st, static_cast<const bf16_t *>(z), part, rows, C, rpc);
        else
            hipLaunchKernelGGL((col_stats_vec_kernel<float, 4>), grid, dim3(256), 0, st, static_cast<const float *>(z), part, rows, C, rpc);
        hipLaunchKernelGGL(col_merge_stats_kernel, dim3(fg), dim3(1024), 0, st, part, nch, C, rows, rpc, eps, mean, var, invstd);
        SOL_HIP(hipGetLastError());
        return SOL_OK;
    }
    if (dt == SOL_BF16) {
        const bf16_t *p = static_cast<const bf16_t *>(z);
        if (C % 8 == 0) hipLaunchKernelGGL((col_reduce_vec_kernel<bf16_t, 8, 0>), grid, dim3(256), 0, st, p, p, p, nullptr, nullptr, part, rows, C, rpc, 0);
        else hipLaunchKernelGGL((col_reduce_kernel<bf16_t, 0>), grid, dim3(256), 0, st, p, p, p, nullptr, nullptr, part, rows, C, rpc, 0);
        hipLaunchKernelGGL(col_finalize_kernel, dim3(fg), dim3(1024), 0, st, part, nch, C, 1.f / rows, mean, nullptr, -1.f, nullptr);
        if (C % 8 == 0) hipLaunchKernelGGL((col_reduce_vec_kernel<bf16_t, 8, 1>), grid, dim3(256), 0, st, p, p, p, mean, nullptr, part, rows, C, rpc, 0);
        else hipLaunchKernelGGL((col_reduce_kernel<bf16_t, 1>), grid, dim3(256), 0, st, p, p, p, mean, nullptr, part, rows, C, rpc, 0);
    } else {
        const float *p = static_cast<const float *>(z);
        if (C % 4 == 0) hipLaunchKernelGGL((col_reduce_vec_kernel<float, 4, 0>), grid, dim3(256), 0, st, p, p, p, nullptr, nullptr, part, rows, C, rpc, 0);
        else hipLaunchKernelGGL((col_reduce_kernel<float, 0>), grid, dim3(256), 0, st, p, p, p, nullptr, nullptr, part, rows, C, rpc, 0);
        hipLaunchKernelGGL(col_finalize_kernel, dim3(fg), dim3(1024), 0, st, part, nch, C, 1.f / rows, mean, nullptr, -1.f, nullptr);
        if (C % 4 == 0) hipLaunchKernelGGL((col_reduce_vec_kernel<float, 4, 1>), grid, dim3(256), 0, st, p, p, p, mean, nullptr, part, rows, C, rpc, 0);
        else hipLaunchKernelGGL((col_reduce_kernel<float, 1>), grid, dim3(256), 0, st, p, p, p, mean, nullptr, part, rows, C, rpc, 0);
    }
    hipLaunchKernelGGL(col_finalize_kernel, dim3(fg), dim3(1024), 0, st, part, nch, C, 1.f / rows, var, nullptr, eps, invstd);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

sol_status launch_bn_apply(const void *z, const void *res, void *y, const float *mean, const float *invstd,
                           const float *gamma, const float *beta, long total, int C, int relu, int dt, hipStream_t st) {
    SOL_DISPATCH_TV(dt, C, {
        if ((256 * V) % C == 0)
            hipLaunchKernelGGL((bn_apply_kernel<T, V, true>), dim3(grid_for(total / V)), dim3(256), 0, st, static_cast<const T *>(z),
                               static_cast<const T *>(res), static_cast<T *>(y), mean, invstd, gamma, beta, total / V, C, relu);
        else
            hipLaunchKernelGGL((bn_apply_kernel<T, V, false>), dim3(grid_for(total / V)), dim3(256), 0, st, static_cast<const T *>(z),
                               static_cast<const T *>(res), static_cast<T *>(y), mean, invstd, gamma, beta, total / V, C, relu);
    });
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

// s0 -> out0 = sum g, s1 -> out1 = sum g xhat  (z may be NULL: out1 unused)
sol_status launch_grad_col_sums(const void *z, const void *dy, const void *y, const float *mean, const float *invstd,
                                int rows, int C, int relu, int dt, float *out0, float *out1, float *part, hipStream_t st) {
    int rpc;
    const int nch = col_reduce_chunks(rows, &rpc);
    const dim3 grid(nch, ceil_div(C, 64));
    if (dt == SOL_BF16 && C % 8 == 0)
        hipLaunchKernelGGL((col_reduce_vec_kernel<bf16_t, 8, 2>), grid, dim3(256), 0, st, static_cast<const bf16_t *>(z),
                           static_cast<const bf16_t *>(dy), static_cast<const bf16_t *>(y), mean, invstd, part, rows, C, rpc, relu);
    else if (dt == SOL_BF16)
        hipLaunchKernelGGL((col_reduce_kernel<bf16_t, 2>), grid, dim3(256), 0, st, static_cast<const bf16_t *>(z),
                           static_cast<const bf16_t *>(dy), static_cast<const bf16_t *>(y), mean, invstd, part, rows, C, rpc, relu);
    else if (C % 4 == 0)
        hipLaunchKernelGGL((col_reduce_vec_kernel<float, 4, 2>), grid, dim3(256), 0, st, static_cast<const float *>(z),
                           static_cast<const float *>(dy), static_cast<const float *>(y), mean, invstd, part, rows, C, rpc, relu);
    else
        hipLaunchKernelGGL((col_reduce_kernel<float, 2>), grid, dim3(256), 0, st, static_cast<const float *>(z),
                           static_cast<const float *>(dy), static_cast<const float *>(y), mean, invstd, part, rows, C, rpc, relu);
    hipLaunchKernelGGL(col_finalize_kernel, dim3(ceil_div(C, 64)), dim3(1024), 0, st, part, nch, C, 1.f, out0, out1, -1.f, nullptr);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

sol_status launch_act_bn_bwd(const void *z, const void *dy, const void *y, const float *mean, const float *invstd,
                             const float *gamma, const float *dbeta, const float *dgamma, void *dz, void *dres,
                             int res_first, long total, int C, int relu, int bn, int rows, int dt, hipStream_t st) {
    SOL_DISPATCH_TV(dt, C, {
        if ((256 * V) % C == 0)
            hipLaunchKernelGGL((act_bn_bwd_kernel<T, V, true>), dim3(grid_for(total / V)), dim3(256), 0, st,
                               static_cast<const T *>(z), static_cast<const T *>(dy), static_cast<const T *>(y), mean, invstd, gamma,
                               dbeta, dgamma, static_cast<T *>(dz), static_cast<T *>(dres), res_first, total / V, C, relu, bn, 1.f / rows);
        else
            hipLaunchKernelGGL((act_bn_bwd_kernel<T, V, false>), dim3(grid_for(total / V)), dim3(256), 0, st,
                               static_cast<const T *>(z), static_cast<const T *>(dy), static_cast<const T *>(y), mean, invstd, gamma,
                               dbeta, dgamma, static_cast<T *>(dz), static_cast<T *>(dres), res_first, total / V, C, relu, bn, 1.f / rows);
    });
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

sol_status launch_dilate(const void *dz, void *out, int N, int Ho, int Wo, int K, int Hd, int Wd, int sh, int sw, int dt,
                         hipStream_t st) {
    const long total = (long)N * Hd * Wd * K;
    SOL_DISPATCH_TV(dt, K, hipLaunchKernelGGL((dilate_kernel<T, V>), dim3(grid_for(total / V)), dim3(256), 0, st,
                                              static_cast<const T *>(dz), static_cast<T *>(out), N, Ho, Wo, K, Hd, Wd, sh, sw));
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

sol_status launch_pool_bwd(const PoolArgs &a, const void *dy, void *dx, int first, int dt, hipStream_t st) {
    const long total = (long)a.N * a.H * a.W * a.C;
    SOL_DISPATCH_TV(dt, a.C, hipLaunchKernelGGL((pool_bwd_kernel<T, V>), dim3(grid_for(total / V)), dim3(256), 0, st, a,
                                                static_cast<const T *>(dy), static_cast<T *>(dx), first));
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

sol_status launch_gap_bwd(const void *dy, void *dx, int N, int HW, int C, int first, int dt, hipStream_t st) {
    const long total = (long)N * HW * C;
    SOL_DISPATCH_TV(dt, C, hipLaunchKernelGGL((gap_bwd_kernel<T, V>), dim3(grid_for(total / V)), dim3(256), 0, st,
                                              static_cast<const T *>(dy), static_cast<T *>(dx), N, HW, C, first));
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

// row_loss: N floats of scratch
sol_status launch_softmax_ce(const void *logits, const int32_t *labels, void *dlogits, float *row_loss, float *loss, int N,
                             int C, int dt, hipStream_t st) {
    if (dt == SOL_BF16)
        hipLaunchKernelGGL((softmax_ce_kernel<bf16_t>), dim3(N), dim3(256), 0, st, static_cast<const bf16_t *>(logits), labels,
                           static_cast<bf16_t *>(dlogits), row_loss, N, C);
    else
        hipLaunchKernelGGL((softmax_ce_kernel<float>), dim3(N), dim3(256), 0, st, static_cast<const float *>(logits), labels,
                           static_cast<float *>(dlogits), row_loss, N, C);
    hipLaunchKernelGGL(loss_mean_kernel, dim3(1), dim3(64), 0, st, row_loss, N, loss);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

sol_status launch_sgd_batch(const SgdBatch &b, float lr, float mu, hipStream_t st) {
    if (b.nseg <= 0 || b.first_block[b.nseg] <= 0) return SOL_OK;
    hipLaunchKernelGGL(sgd_batch_kernel, dim3(b.first_block[b.nseg]), dim3(256), 0, st, b, lr, mu);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

sol_status launch_pack_batch(const PackBatch &b, int dt, hipStream_t st) {
    if (b.nseg <= 0 || b.first_block[b.nseg] <= 0) return SOL_OK;
    if (dt == SOL_BF16)
        hipLaunchKernelGGL((pack_batch_kernel<bf16_t>), dim3(b.first_block[b.nseg]), dim3(256), 0, st, b);
    else
        hipLaunchKernelGGL((pack_batch_kernel<float>), dim3(b.first_block[b.nseg]), dim3(256), 0, st, b);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

sol_status launch_pack_flip(const sol_conv_desc &cd, int dt, const float *w, void *packed, hipStream_t st) {
    // cd describes the forward convolution; the packed result belongs to {cout = cin, cin = cout, same filter}
    const sol_conv_desc td{cd.cin, cd.cout, cd.kh, cd.kw, 1, 1, 0, 0};
    const int Kp = packed_k(td, dt);
    const long total = (long)cd.cin * Kp;
    if (dt == SOL_BF16)
        hipLaunchKernelGGL((pack_weights_flip_kernel<bf16_t>), dim3(grid_for(total)), dim3(256), 0, st, w,
                           static_cast<bf16_t *>(packed), cd.cout, cd.cin, cd.kh, cd.kw, Kp);
    else
        hipLaunchKernelGGL((pack_weights_flip_kernel<float>), dim3(grid_for(total)), dim3(256), 0, st, w,
                           static_cast<float *>(packed), cd.cout, cd.cin, cd.kh, cd.kw, Kp);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

// Split of the pixel reduction: enough workgroups to fill the chip, at least 16 steps each.
// bf16 with whole 16-byte slots of channels on both sides: the LDS-staged kernel (steps of 64 pixels)
static bool wgrad_lds_applies(const sol_tensor_desc &xd, const sol_conv_desc &cd) {
    return xd.dtype == SOL_BF16 && cd.cout % 8 == 0 && cd.cin % 8 == 0;
}

// bf16 3x3 / stride 1 / pad 1 with at most 62 pixels per image row: the filter-row kernel (stages of whole image rows)
static bool wgrad_row_applies(const sol_tensor_desc &xd, const sol_conv_desc &cd) {
    return xd.dtype == SOL_BF16 && cd.cout % 8 == 0 && cd.cin % 8 == 0 && cd.kh == 3 && cd.kw == 3 && cd.sh == 1 && cd.sw == 1 &&
           cd.ph == 1 && cd.pw == 1 && xd.w <= 62 && xd.n > 0;
}
static void wgrad_row_plan(const sol_tensor_desc &xd, const sol_conv_desc &cd, int *nr, int *nstages, int *nsplit) {
    *nr = std::max(1, 64 / xd.w);
    *nstages = ceil_div(xd.n * xd.h, *nr);
    const int tiles = ceil_div(cd.cout, 64) * ceil_div(cd.cin, 64) * 3;
    *nsplit = std::max(1, std::min(ceil_div(256, tiles), std::max(1, *nstages / 6)));
}

// bf16 7x7 / stride 2 / pad 3 over 3 input channels, at most 64 output channels: the stem kernel
static bool wgrad_stem_applies(const sol_tensor_desc &xd, const sol_conv_desc &cd) {
    return xd.dtype == SOL_BF16 && xd.c == 3 && cd.cin == 3 && cd.kh == 7 && cd.kw == 7 && cd.sh == 2 && cd.sw == 2 && cd.ph == 3 &&
           cd.pw == 3 && cd.cout <= 64 && cd.cout % 8 == 0;
}
static int wgrad_stem_grid(const sol_tensor_desc &xd, int Ho, int Wo) {
    const long tiles = (long)xd.n * ceil_div(Ho, WS_TH) * ceil_div(Wo, WS_TW);
    return (int)std::min<long>(tiles, 256);
}

void wgrad_plan(const sol_tensor_desc &xd, const sol_conv_desc &cd, int Ho, int Wo, int *nsplit, size_t *part_floats) {
    if (wgrad_stem_applies(xd, cd)) {
        *nsplit = std::max(1, wgrad_stem_grid(xd, Ho, Wo));
        *part_floats = (size_t)*nsplit * cd.cout * 147;
        return;
    }
    if (wgrad_row_applies(xd, cd)) {
        int nr, nst, ns;
        wgrad_row_plan(xd, cd, &nr, &nst, &ns);
        *nsplit = ns;
        *part_floats = (size_t)ns * cd.cout * 9 * cd.cin;
        return;
    }
    if (wgrad_lds_applies(xd, cd)) {
        const int nsteps = (int)(((long)xd.n * Ho * Wo + 63) / 64);
        const int tiles = ceil_div(cd.cout, 64) * ceil_div(cd.cin, 64) * cd.kh * cd.kw;
        int ns = std::max(1, ceil_div(384, tiles));              // 1.5 workgroups per CU measured best (two fit; fewer splits also mean fewer partials)
        ns = std::min(ns, std::max(1, nsteps / 8));
        *nsplit = ns;
        *part_floats = (size_t)ns * cd.cout * cd.kh * cd.kw * cd.cin;
        return;
    }
    const int GP = 16 / (int)dtype_size(xd.dtype);
    const int G = ceil_div(Wo, GP);
    const long ngroups = (long)xd.n * Ho * G;
    const int nsteps = (int)((ngroups + 1) / 2);
    const int tiles = ceil_div(cd.cout, 64) * ceil_div(cd.cin, 64) * cd.kh * cd.kw;
    int ns = std::max(1, ceil_div(1024, tiles));
    ns = std::min(ns, std::max(1, nsteps / 16));
    *nsplit = ns;
    *part_floats = (size_t)ns * cd.cout * cd.kh * cd.kw * cd.cin;
}

// dw: fp32 [cout][cin][kh][kw]; part: scratch of wgrad_plan's size
sol_status launch_wgrad(const sol_tensor_desc &xd, const void *x, const sol_conv_desc &cd, const void *dz, int Ho, int Wo,
                        float *dw, float *part, hipStream_t st, int *deferred_nsplit) {
    WgradArgs a;
    memset(static_cast<void *>(&a), 0, sizeof(a));
    const int ES = (int)dtype_size(xd.dtype), GP = 16 / ES;
    const double xb = (double)xd.n * xd.h * xd.w * xd.c * ES, zb = (double)xd.n * Ho * Wo * cd.cout * ES;
    SOL_REQUIRE(xb < 2147483648.0 && zb < 2147483648.0, SOL_ERR_UNSUPPORTED, "weight gradient: operand of 2 GiB or more");
    a.x = x; a.dz = dz; a.part = part;
    a.N = xd.n; a.H = xd.h; a.W = xd.w; a.C = xd.c; a.K = cd.cout; a.R = cd.kh; a.S = cd.kw;
    a.sh = cd.sh; a.sw = cd.sw; a.ph = cd.ph; a.pw = cd.pw; a.Ho = Ho; a.Wo = Wo;
    if (wgrad_stem_applies(xd, cd)) {
        const int tiles_h = ceil_div(Ho, WS_TH), tiles_w = ceil_div(Wo, WS_TW), ntiles = xd.n * tiles_h * tiles_w;
        size_t pf;
        wgrad_plan(xd, cd, Ho, Wo, &a.nsplit, &pf);
        a.dz_bytes = (uint32_t)zb; a.x_bytes = (uint32_t)xb;
        if (ntiles > 0) {
            hipLaunchKernelGGL(wgrad_stem_kernel, dim3(a.nsplit), dim3(256), 0, st, a, tiles_h, tiles_w, ntiles);
            const long total = (long)cd.cout * 147;
            if (!deferred_nsplit)
                hipLaunchKernelGGL(wgrad_reduce_kernel, dim3(grid_for(total)), dim3(256), 0, st, part, a.nsplit, dw, cd.cout, cd.cin, 49);
        }
        if (deferred_nsplit) *deferred_nsplit = ntiles > 0 ? a.nsplit : 0;
        SOL_HIP(hipGetLastError());
        return SOL_OK;
    }
    if (wgrad_row_applies(xd, cd)) {
        int nr;
        wgrad_row_plan(xd, cd, &nr, &a.nsteps, &a.nsplit);
        a.steps_per_split = ceil_div(a.nsteps, a.nsplit);
        a.nkt = ceil_div(cd.cout, 64); a.nct = ceil_div(cd.cin, 64);
        a.x_bytes = (uint32_t)xb; a.dz_bytes = (uint32_t)zb;
        hipLaunchKernelGGL(wgrad_row_kernel, dim3(a.nkt * a.nct * 3 * a.nsplit), dim3(256), 0, st, a, nr);
        if (deferred_nsplit)
            *deferred_nsplit = a.nsplit;
        else
            hipLaunchKernelGGL(wgrad_reduce_kernel, dim3(grid_for((long)cd.cout * 9 * cd.cin)), dim3(256), 0, st, part, a.nsplit, dw,
                               cd.cout, cd.cin, 9);
        SOL_HIP(hipGetLastError());
        return SOL_OK;
    }
    const bool lds_path = wgrad_lds_applies(xd, cd);
    a.G = lds_path ? Wo : ceil_div(Wo, GP);
    a.ngroups = xd.n * Ho * a.G;
    a.nsteps = lds_path ? (int)(((long)xd.n * Ho * Wo + 63) / 64) : (a.ngroups + 1) / 2;
    size_t pf;
    wgrad_plan(xd, cd, Ho, Wo, &a.nsplit, &pf);
    a.steps_per_split = ceil_div(a.nsteps, a.nsplit);
    a.nkt = ceil_div(cd.cout, 64); a.nct = ceil_div(cd.cin, 64);
    a.x_bytes = (uint32_t)xb; a.dz_bytes = (uint32_t)zb;
    a.dG = FastDiv((uint32_t)a.G); a.dHo = FastDiv((uint32_t)Ho);
    const int grid = a.nkt * a.nct * cd.kh * cd.kw * a.nsplit;
    if (lds_path)
        hipLaunchKernelGGL((wgrad_lds_kernel<4>), dim3(grid), dim3(256), 0, st, a);
    else if (xd.dtype == SOL_BF16)
        hipLaunchKernelGGL((wgrad_kernel<bf16_t>), dim3(grid), dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL((wgrad_kernel<float>), dim3(grid), dim3(256), 0, st, a);
    const long total = (long)cd.cout * cd.kh * cd.kw * cd.cin;
    if (deferred_nsplit)
        *deferred_nsplit = a.nsplit;
    else
        hipLaunchKernelGGL(wgrad_reduce_kernel, dim3(grid_for(total)), dim3(256), 0, st, part, a.nsplit, dw, cd.cout, cd.cin,
                           cd.kh * cd.kw);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

}  // namespace sol

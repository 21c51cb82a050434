// Device-side pieces shared by the convolution kernels (internal): MFMA wrappers, the GEMM-row ->
// pixel map, 8-channel vector access, and the fused epilogue.
#pragma once
#include <type_traits>

#include "common.h"

namespace sol {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

template <typename T> struct Mma;
template <> struct Mma<bf16_t> {
    // one v_mfma_f32_32x32x16_bf16: each lane supplies 8 consecutive reduction elements
    template <typename V> static __device__ __forceinline__ void run(f32x16_t &acc, const V &a, const V &b) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                      __builtin_bit_cast(bf16x8_t, b), acc, 0, 0, 0);
    }
};
template <> struct Mma<float> {
    // four v_mfma_f32_32x32x2_f32 (true fp32 multiplies); the reduction order inside a 128-byte row
    // is permuted identically for both operands, which leaves the sum unchanged
    template <typename V> static __device__ __forceinline__ void run(f32x16_t &acc, const V &a, const V &b) {
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
    }
};

// Hand-ordered LDS pipeline pieces shared by the DMA-ring kernels.  The compiler cannot tell which ring stage an
// LDS read touches and would make every fragment read wait for all outstanding DMA; the reads are therefore opaque
// volatile statements ordered by hand (ds_read -> s_waitcnt lgkmcnt -> landed() -> use).
namespace lds_pipe {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;

template <int N> __device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
template <int N> __device__ __forceinline__ void wait_lgkmcnt() { asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory"); }
template <int OFF> __device__ __forceinline__ void lds_read16(u32x4_t &dst, unsigned addr) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(dst) : "v"(addr), "n"(OFF));
}
// ties a fragment to a point after the wait: every later use depends on it
__device__ __forceinline__ void landed(u32x4_t &v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ unsigned lds_addr(const void *p) {
    return (unsigned)(size_t)(__attribute__((address_space(3))) const void *)p;
}
// (a ^ x) + b in one VALU instruction, opaque to the optimiser: fragment addresses are derived from one base per
// row at the point of use instead of being hoisted into dozens of loop-invariant registers
__device__ __forceinline__ unsigned xor_add(unsigned a, unsigned x, unsigned b) {
    unsigned d;
    asm volatile("v_xad_u32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "s"(x), "v"(b));
    return d;
}
// 16-byte slot permutation of a tile row (applied to the global address a DMA lane fetches): conflict-free
// 16-byte fragment reads for rows of 128 bytes (8 slots) and of 64 bytes (4 slots)
template <int ROWB> __device__ __forceinline__ int swz(int row) { return ROWB == 256 ? (row & 15) : ROWB == 128 ? ((row >> 1) & 7) : ((row >> 2) & 3); }

}  // namespace lds_pipe

// Warms this XCD's L2 with a range of the layer's packed weights.  Inside a network the weights of a layer are
// cold when it starts, every workgroup streams the same rows in lock step, and each stage would stall on an HBM
// round trip; instead the workgroups of an XCD (blockIdx & 7) touch one dword per 128-byte line of the range
// between them at kernel entry, all misses in flight at once.  The touched dwords are dropped into a per-wave LDS
// sink of 256 bytes (a load into a register would have to be waited for, a DMA does not).
__device__ __forceinline__ void warm_l2(const unsigned char *base, unsigned bytes, unsigned char *sink_wave, int tid, int nthreads) {
    const unsigned nx = gridDim.x >> 3, lines = bytes >> 7;
    for (unsigned l = (blockIdx.x >> 3) * nthreads + tid; l < lines; l += nx * nthreads)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(base + ((size_t)l << 7)),
                                         (__attribute__((address_space(3))) void *)sink_wave, 4, 0, 0);
}

// GEMM row m -> output pixel.  With a fused 2x2 pool the rows are ordered window-major, so that the
// four elements of one pooling window sit in four adjacent lanes in row-major window order.
__device__ __forceinline__ void decode_pixel(const ConvArgs &a, int m, int &n, int &op, int &oq) {
    uint32_t t, x, nn, y;
    a.dw.divmod((uint32_t)(a.pool ? m >> 2 : m), t, x);     // x = column (of the window / of the pixel)
    a.dh.divmod(t, nn, y);
    n = (int)nn;
    if (a.pool) {
        const int d = m & 3;
        op = 2 * (int)y + (d >> 1);
        oq = 2 * (int)x + (d & 1);
    } else {
        op = (int)y;
        oq = (int)x;
    }
}

template <typename T> __device__ __forceinline__ void store_vec8(T *p, const float v[8]);
template <> __device__ __forceinline__ void store_vec8<float>(float *p, const float v[8]) {
    reinterpret_cast<float4 *>(p)[0] = make_float4(v[0], v[1], v[2], v[3]);
    reinterpret_cast<float4 *>(p)[1] = make_float4(v[4], v[5], v[6], v[7]);
}
template <> __device__ __forceinline__ void store_vec8<bf16_t>(bf16_t *p, const float v[8]) {
    uint4 u;
    u.x = pack_bf16x2(v[0], v[1]);
    u.y = pack_bf16x2(v[2], v[3]);
    u.z = pack_bf16x2(v[4], v[5]);
    u.w = pack_bf16x2(v[6], v[7]);
    *reinterpret_cast<uint4 *>(p) = u;
}
template <typename T> __device__ __forceinline__ void load_vec8(const T *p, float v[8]);
template <> __device__ __forceinline__ void load_vec8<float>(const float *p, float v[8]) {
    const float4 f = reinterpret_cast<const float4 *>(p)[0], g = reinterpret_cast<const float4 *>(p)[1];
    v[0] = f.x; v[1] = f.y; v[2] = f.z; v[3] = f.w; v[4] = g.x; v[5] = g.y; v[6] = g.z; v[7] = g.w;
}
template <> __device__ __forceinline__ void load_vec8<bf16_t>(const bf16_t *p, float v[8]) {
    const uint4 u = *reinterpret_cast<const uint4 *>(p);
    v[0] = __uint_as_float(u.x << 16); v[1] = __uint_as_float(u.x & 0xffff0000u);
    v[2] = __uint_as_float(u.y << 16); v[3] = __uint_as_float(u.y & 0xffff0000u);
    v[4] = __uint_as_float(u.z << 16); v[5] = __uint_as_float(u.z & 0xffff0000u);
    v[6] = __uint_as_float(u.w << 16); v[7] = __uint_as_float(u.w & 0xffff0000u);
}

// nv = number of valid channels among the 8 (<= 0: none); vec = Cout % 8 == 0 (aligned, never ragged)
template <typename T>
__device__ __forceinline__ void store8(T *p, const float v[8], int nv, bool vec) {
    if (vec) { store_vec8<T>(p, v); return; }
#pragma unroll
    for (int e = 0; e < 8; e++)
        if (e < nv) Elem<T>::store(p + e, v[e]);
}
template <typename T>
__device__ __forceinline__ void load8(const T *p, float v[8], int nv, bool vec) {
    if (vec) { load_vec8<T>(p, v); return; }
#pragma unroll
    for (int e = 0; e < 8; e++) v[e] = e < nv ? Elem<T>::load(p + e) : 0.f;
}

template <int N, int I = 0, typename F> __device__ __forceinline__ void static_for(F &&f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<N, I + 1>(f);
    }
}

// Fused epilogue shared by all convolution kernels.  acc[i][j] is the 32x32 accumulator block of
// channel block i and pixel block j of this wave (MFMA layout: lane = pixel, 4-register groups =
// 4 consecutive channels).  lds_f: LDS scratch of at least NW*32*(TC*32+4) floats that no wave still
// reads as tile data (each wave uses a private strip of it, so the epilogue needs no workgroup barrier); mw / cw: first GEMM row / first output channel of this wave's tile.
// rowmap(m): output pixel index of tile row m (counted from mw), or -1 if the row is padding; only
// consulted when no pool is fused (the fused pool relies on the window-major GEMM row order).
struct LinearRows {
    int P;
    __device__ __forceinline__ long operator()(int m) const { return m < P ? (long)m : -1L; }
};

// Orders this wave's earlier LDS accesses before its later ones (wave-private scratch: the LDS unit
// executes one wave's instructions in order, so only the compiler has to be kept from reordering).
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Per-lane affine map of the epilogue (folded BN + bias of this lane's 8 output channels).  Loaded
// ahead of the main loop so that the latency of these loads is hidden behind it.
struct Affine8 {
    float sc[8], sf[8];
};
template <int TC> __device__ __forceinline__ Affine8 load_affine(const ConvArgs &a, int lane, int cw) {
    const int cb = cw + (lane % (TC * 4)) * 8;
    const int nv = min(8, a.Cout - cb);
    Affine8 f;
    if (nv == 8 && a.scale && a.shift) {          // the usual case: two aligned 32-byte runs
        const float4 s0 = *reinterpret_cast<const float4 *>(a.scale + cb), s1 = *reinterpret_cast<const float4 *>(a.scale + cb + 4);
        const float4 h0 = *reinterpret_cast<const float4 *>(a.shift + cb), h1 = *reinterpret_cast<const float4 *>(a.shift + cb + 4);
        f.sc[0] = s0.x; f.sc[1] = s0.y; f.sc[2] = s0.z; f.sc[3] = s0.w; f.sc[4] = s1.x; f.sc[5] = s1.y; f.sc[6] = s1.z; f.sc[7] = s1.w;
        f.sf[0] = h0.x; f.sf[1] = h0.y; f.sf[2] = h0.z; f.sf[3] = h0.w; f.sf[4] = h1.x; f.sf[5] = h1.y; f.sf[6] = h1.z; f.sf[7] = h1.w;
        return f;
    }
#pragma unroll
    for (int e = 0; e < 8; e++) {
        f.sc[e] = (a.scale && e < nv) ? a.scale[cb + e] : 1.f;
        f.sf[e] = (a.shift && e < nv) ? a.shift[cb + e] : 0.f;
    }
    return f;
}

// Branch-free variant for kernels whose launcher guarantees scale and shift are present and Cout % 8 == 0:
// four unconditional 16-byte loads (lanes of a ragged channel tile read channel 0 and never use the values),
// so that the compiler has no reason to wait for them before the first use in the epilogue.
template <int TC> __device__ __forceinline__ Affine8 load_affine_unconditional(const ConvArgs &a, int lane, int cw) {
    int cb = cw + (lane % (TC * 4)) * 8;
    cb = cb + 8 <= a.Cout ? cb : 0;
    const float4 s0 = *reinterpret_cast<const float4 *>(a.scale + cb), s1 = *reinterpret_cast<const float4 *>(a.scale + cb + 4);
    const float4 h0 = *reinterpret_cast<const float4 *>(a.shift + cb), h1 = *reinterpret_cast<const float4 *>(a.shift + cb + 4);
    Affine8 f;
    f.sc[0] = s0.x; f.sc[1] = s0.y; f.sc[2] = s0.z; f.sc[3] = s0.w; f.sc[4] = s1.x; f.sc[5] = s1.y; f.sc[6] = s1.z; f.sc[7] = s1.w;
    f.sf[0] = h0.x; f.sf[1] = h0.y; f.sf[2] = h0.z; f.sf[3] = h0.w; f.sf[4] = h1.x; f.sf[5] = h1.y; f.sf[6] = h1.z; f.sf[7] = h1.w;
    return f;
}

// Residual rows of a wave's tile, fetched into registers ahead of the main loop (same lane -> 8-channel
// mapping as the epilogue's output rows), so that their HBM latency overlaps the tile loads instead
// of following them.  Only used without a fused pool and when rows are 16-byte aligned.
template <typename T> struct Raw8;
template <> struct Raw8<bf16_t> {
    uint4 v;
    __device__ __forceinline__ void load(const bf16_t *p) { v = *reinterpret_cast<const uint4 *>(p); }
    __device__ __forceinline__ void get(float f[8]) const {
        f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
        f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
        f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
        f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
    }
};
template <> struct Raw8<float> {
    float4 lo, hi;
    __device__ __forceinline__ void load(const float *p) {
        lo = reinterpret_cast<const float4 *>(p)[0]; hi = reinterpret_cast<const float4 *>(p)[1];
    }
    __device__ __forceinline__ void get(float f[8]) const {
        f[0] = lo.x; f[1] = lo.y; f[2] = lo.z; f[3] = lo.w; f[4] = hi.x; f[5] = hi.y; f[6] = hi.z; f[7] = hi.w;
    }
};
template <typename T, int TP, int TC> struct ResidualRegs {
    static constexpr int PASSES = 32 / (64 / (TC * 4));
    Raw8<T> r[TP][PASSES];
    bool on;
};
template <typename T, int TP, int TC, typename RowMap>
__device__ __forceinline__ void prefetch_residual(const ConvArgs &a, int lane, int mw, int cw, const RowMap &rowmap,
                                                  ResidualRegs<T, TP, TC> &out) {
    constexpr int LPR = TC * 4, RPS = 64 / LPR;
    const T *__restrict__ resg = static_cast<const T *>(a.res);
    const int cb = cw + (lane % LPR) * 8, erow = lane / LPR;
    out.on = resg != nullptr && a.pool == 0 && (a.Cout & 7) == 0;
    if (!out.on) return;
#pragma unroll
    for (int j = 0; j < TP; j++)
#pragma unroll
        for (int ps = 0; ps < 32 / RPS; ps++) {
            const long m = rowmap(mw + j * 32 + erow + ps * RPS);
            if (m >= 0 && cb < a.Cout) out.r[j][ps].load(resg + m * a.Cout + cb);
        }
}

template <typename T, int TP, int TC, typename RowMap>
__device__ __forceinline__ void conv_epilogue(const ConvArgs &a, f32x16_t (&acc)[TC][TP], float *lds_f, int wave,
                                              int lane, int mw, int cw, const Affine8 &aff, const RowMap &rowmap,
                                              const ResidualRegs<T, TP, TC> &pre) {
    const int lr = lane & 31, lh = lane >> 5;
    // ---- fused epilogue: affine (folded BN + bias), residual, activation, optional 2x2 pool -------
    // The accumulators hold 4 channels x 1 pixel per lane; writing them out directly would give
    // 8-byte stores scattered over 32 pixel rows.  Each wave therefore transposes one 32-pixel block
    // at a time through a private LDS strip and writes rows of 8 channels per lane: whole 128-byte
    // lines for the output and the residual alike.
    constexpr int ECH = TC * 32;                 // channels per wave
    constexpr int ERS = ECH + 4;                 // padded strip row, in floats
    constexpr int LPR = ECH / 8;                 // lanes per pixel row (8 channels each)
    constexpr int RPS = 64 / LPR;                // pixel rows per pass
    float *strip = lds_f + wave * (32 * ERS);
    T *__restrict__ yg = static_cast<T *>(a.y);
    const T *__restrict__ resg = static_cast<const T *>(a.res);
    T *__restrict__ preg = static_cast<T *>(a.prepool);
    const int ecg = lane % LPR, erow = lane / LPR;
    const int cb = cw + ecg * 8;                  // first of this lane's 8 output channels
    const int nv = min(8, a.Cout - cb);          // how many of them exist
    const bool vec = (a.Cout & 7) == 0;          // rows are 16-byte aligned and never ragged
    const float *sc = aff.sc, *sf = aff.sf;
    auto finish_row = [&](int row, long opix, float v[8], const Raw8<T> *pr = nullptr) {   // strip row -> act(scale*acc + shift + residual)
        const float4 lo = *reinterpret_cast<const float4 *>(strip + row * ERS + ecg * 8);
        const float4 hi = *reinterpret_cast<const float4 *>(strip + row * ERS + ecg * 8 + 4);
        const float r[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
        for (int e = 0; e < 8; e++) v[e] = r[e] * sc[e] + sf[e];
        if (pr) {
            float rv[8];
            pr->get(rv);
#pragma unroll
            for (int e = 0; e < 8; e++) v[e] += rv[e];
        } else if (resg) {
            float rv[8];
            load8<T>(resg + opix * a.Cout + cb, rv, nv, vec);
#pragma unroll
            for (int e = 0; e < 8; e++) v[e] += rv[e];
        }
        if (a.act == SOL_ACT_RELU) {
#pragma unroll
            for (int e = 0; e < 8; e++) v[e] = __builtin_fmaxf(v[e], 0.f);     // one v_max: a NaN becomes 0, as with a compare and a select
        }
    };
    // compile-time loop over the pixel blocks: the accumulator index must be a constant
    static_for<TP>([&](auto J) {
        constexpr int j = decltype(J)::value;
        const int mb = mw + j * 32;          // first GEMM row of this 32-pixel block
#pragma unroll
        for (int i = 0; i < TC; i++)
#pragma unroll
            for (int g = 0; g < 4; g++)
                *reinterpret_cast<float4 *>(strip + lr * ERS + i * 32 + 8 * g + 4 * lh) =
                    make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
        wave_lds_fence();
        if (!a.pool) {
#pragma unroll
            for (int ps = 0; ps < 32 / RPS; ps++) {
                const int row = erow + ps * RPS;
                const long m = rowmap(mb + row);        // output pixel index, or -1
                if (m >= 0 && nv > 0) {
                    float v[8];
                    finish_row(row, m, v, pre.on ? &pre.r[j][ps] : nullptr);
                    store8<T>(yg + m * a.ldy + cb, v, nv, vec);
                }
            }
        } else {
            // rows 4w..4w+3 of the strip are the 4 elements of pooling window w, in row-major window order
            for (int w = erow; w < 8; w += RPS) {
                const int m0 = mb + 4 * w;
                if (m0 < a.P && nv > 0) {
                    int n, op, oq;
                    decode_pixel(a, m0, n, op, oq);                 // top-left element of the window
                    float best[8];
                    int bi[8];
#pragma unroll
                    for (int d = 0; d < 4; d++) {
                        const long opix = ((long)n * a.Ho + op + (d >> 1)) * a.Wo + oq + (d & 1);
                        float v[8];
                        finish_row(4 * w + d, opix, v);
                        if (preg) store8<T>(preg + opix * a.Cout + cb, v, nv, vec);
#pragma unroll
                        for (int e = 0; e < 8; e++) {
                            if (a.pool == 1) {          // strict '>' in scan order: the first maximum wins
                                if (d == 0 || v[e] > best[e]) { best[e] = v[e]; bi[e] = d; }
                            } else {
                                best[e] = d == 0 ? v[e] : best[e] + v[e];
                            }
                        }
                    }
                    if (a.pool == 2) {
#pragma unroll
                        for (int e = 0; e < 8; e++) best[e] *= 0.25f;
                    }
                    const long obase = (long)(m0 >> 2) * a.Cout + cb;
                    store8<T>(yg + obase, best, nv, vec);
                    if (a.argmax && a.pool == 1) {
#pragma unroll
                        for (int e = 0; e < 8; e++)
                            if (e < nv) a.argmax[obase + e] = (op + (bi[e] >> 1)) * a.Wo + oq + (bi[e] & 1);
                    }
                }
            }
        }
        wave_lds_fence();
    });
}

// Epilogue fast path for a wave tile that lies completely inside the output (all TP*32 rows below P, all TC*32
// channels below Cout), Cout % 8 == 0 and no fused pool: same transposition through the wave-private strip as
// conv_epilogue, but without per-row / per-channel range logic, with 32-bit element offsets (tensors are
// limited to < 2^31 elements) and a select for the activation (same NaN behaviour as conv_epilogue).  RES: add the prefetched residual rows.
// rowoff(r): element offset of the first channel of the output pixel of tile row r (counted from the wave's first
// row); rows r .. r + RPS - 1 handled by one pass need not be contiguous with the next pass.
struct LinearRowOffset {
    unsigned first, cout;
    __device__ __forceinline__ unsigned operator()(int r) const { return first + (unsigned)r * cout; }
    __device__ __forceinline__ bool valid(int) const { return true; }     // every row of an interior tile is stored
    // offset of row lane_row + r as a per-lane part, computed once, plus a wave-uniform part (no multiply per store)
    __device__ __forceinline__ unsigned lane_base(int lane_row) const { return first + (unsigned)lane_row * cout; }
    __device__ __forceinline__ unsigned at(unsigned lb, int r) const { return lb + (unsigned)r * cout; }
};
template <typename T, int TP, int TC, bool RES, typename RowOff>
__device__ __forceinline__ void conv_epilogue_interior(const ConvArgs &a, f32x16_t (&acc)[TC][TP], float *lds_f, int wave, int lane,
                                                       int cw, const Affine8 &aff, const ResidualRegs<T, TP, TC> &pre,
                                                       const RowOff &rowoff) {
    constexpr int ECH = TC * 32, ERS = ECH + 4, LPR = ECH / 8, RPS = 64 / LPR;
    const int lr = lane & 31, lh = lane >> 5;
    float *strip = lds_f + wave * (32 * ERS);
    T *__restrict__ yg = static_cast<T *>(a.y);
    const int ecg = lane % LPR, erow = lane / LPR;
    const float lim = a.act == SOL_ACT_RELU ? 0.f : __builtin_nanf("");     // wave-uniform lower bound of the outputs (none: NaN)
    const unsigned coff = (unsigned)(cw + ecg * 8);
    const unsigned lb = rowoff.lane_base(erow);
    constexpr int NPS = 32 / RPS;
    auto write_block = [&](auto J) {                       // accumulator blocks of pixel block j -> strip rows
        constexpr int j = decltype(J)::value;
#pragma unroll
        for (int i = 0; i < TC; i++)
#pragma unroll
            for (int g = 0; g < 4; g++)
                *reinterpret_cast<float4 *>(strip + lr * ERS + i * 32 + 8 * g + 4 * lh) =
                    make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
    };
    write_block(std::integral_constant<int, 0>{});
    wave_lds_fence();
    static_for<TP>([&](auto J) {
        constexpr int j = decltype(J)::value;
        // all rows of the block into registers first; the strip is then free for the next block, whose way to LDS overlaps
        // this block's arithmetic and stores (a wave's epilogue is a chain of LDS round trips: one less per block)
        float4 lo[NPS], hi[NPS];
#pragma unroll
        for (int ps = 0; ps < NPS; ps++) {
            const float *src = strip + (erow + ps * RPS) * ERS + ecg * 8;
            lo[ps] = *reinterpret_cast<const float4 *>(src);
            hi[ps] = *reinterpret_cast<const float4 *>(src + 4);
        }
        wave_lds_fence();
        if constexpr (j + 1 < TP) write_block(std::integral_constant<int, j + 1>{});
#pragma unroll
        for (int ps = 0; ps < NPS; ps++) {
            const float r[8] = {lo[ps].x, lo[ps].y, lo[ps].z, lo[ps].w, hi[ps].x, hi[ps].y, hi[ps].z, hi[ps].w};
            float v[8];
#pragma unroll
            for (int e = 0; e < 8; e++) v[e] = r[e] * aff.sc[e] + aff.sf[e];
            if constexpr (RES) {
                float rv[8];
                pre.r[j][ps].get(rv);
#pragma unroll
                for (int e = 0; e < 8; e++) v[e] += rv[e];
            }
#pragma unroll
            for (int e = 0; e < 8; e++) v[e] = __builtin_fmaxf(v[e], lim);   // one v_max; as the general epilogue: NaN stays NaN without ReLU (the maximum with a NaN is the other operand), ReLU maps it to 0
            if (rowoff.valid(j * 32 + erow + ps * RPS)) store_vec8<T>(yg + rowoff.at(lb, j * 32 + ps * RPS) + coff, v);
        }
        wave_lds_fence();
    });
}

// Chooses the interior fast path when the wave tile allows it (wave-uniform decision), else the general epilogue.
template <typename T, int TP, int TC, typename RowMap>
__device__ __forceinline__ void conv_epilogue_auto(const ConvArgs &a, f32x16_t (&acc)[TC][TP], float *lds_f, int wave, int lane,
                                                   int mw, int cw, const Affine8 &aff, const RowMap &rowmap,
                                                   const ResidualRegs<T, TP, TC> &pre) {
    const bool interior = a.pool == 0 && (a.Cout & 7) == 0 && mw + TP * 32 <= a.P && cw + TC * 32 <= a.Cout;
    const LinearRowOffset ro{(unsigned)mw * (unsigned)a.ldy, (unsigned)a.ldy};
    if (interior && a.res == nullptr) conv_epilogue_interior<T, TP, TC, false>(a, acc, lds_f, wave, lane, cw, aff, pre, ro);
    else if (interior && pre.on) conv_epilogue_interior<T, TP, TC, true>(a, acc, lds_f, wave, lane, cw, aff, pre, ro);
    else conv_epilogue<T, TP, TC>(a, acc, lds_f, wave, lane, mw, cw, aff, rowmap, pre);
}

}  // namespace sol

// V consecutive channel elements of one pixel <-> fp32 registers (V * sizeof(T) = 16 bytes, or V = 1
// for channel counts that do not divide).  Shared by the memory-bound kernels.
#pragma once
#include "common.h"

namespace sol {

template <typename T, int V> struct VecIO;
template <> struct VecIO<float, 4> {
    static __device__ __forceinline__ void load(const float *p, float v[4]) {
        const float4 f = *reinterpret_cast<const float4 *>(p);
        v[0] = f.x; v[1] = f.y; v[2] = f.z; v[3] = f.w;
    }
    static __device__ __forceinline__ void unpack(const uint4 &u, float v[4]) {
        v[0] = __uint_as_float(u.x); v[1] = __uint_as_float(u.y); v[2] = __uint_as_float(u.z); v[3] = __uint_as_float(u.w);
    }
    static __device__ __forceinline__ void store(float *p, const float v[4]) {
        *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    }
};
template <> struct VecIO<float, 1> {
    static __device__ __forceinline__ void unpack(const uint4 &u, float v[1]) { v[0] = __uint_as_float(u.x); }
    static __device__ __forceinline__ void load(const float *p, float v[1]) { v[0] = *p; }
    static __device__ __forceinline__ void store(float *p, const float v[1]) { *p = v[0]; }
};
template <> struct VecIO<bf16_t, 8> {
    static __device__ __forceinline__ void load(const bf16_t *p, float v[8]) { unpack(*reinterpret_cast<const uint4 *>(p), v); }
    static __device__ __forceinline__ void unpack(const uint4 &u, float v[8]) {
        const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; i++) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ void store(bf16_t *p, const float v[8]) {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; i++) w[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
        *reinterpret_cast<uint4 *>(p) = make_uint4(w[0], w[1], w[2], w[3]);
    }
};
template <> struct VecIO<bf16_t, 1> {
    static __device__ __forceinline__ void unpack(const uint4 &u, float v[1]) { v[0] = bf16_to_f32((bf16_t)u.x); }
    static __device__ __forceinline__ void load(const bf16_t *p, float v[1]) { v[0] = bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(bf16_t *p, const float v[1]) { *p = f32_to_bf16(v[0]); }
};

}  // namespace sol

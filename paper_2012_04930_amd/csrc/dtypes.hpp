// Storage types of features and activations: float32 or bfloat16 (round to nearest even on store,
// exact widening on load).  Arithmetic is always float32.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace gcn {

typedef __bf16 bf16_t;

// Number of elements in one 16-byte piece
template <typename T>
struct Piece;
template <>
struct Piece<float> {
    static constexpr int kElems = 4;
};
template <>
struct Piece<bf16_t> {
    static constexpr int kElems = 8;
};

__device__ inline float widen(float v) { return v; }
__device__ inline float widen(bf16_t v) { return (float)v; }

template <typename T>
__device__ inline T narrow(float v);
template <>
__device__ inline float narrow<float>(float v) {
    return v;
}
template <>
__device__ inline bf16_t narrow<bf16_t>(float v) {
    return (bf16_t)v;   // v_cvt_pk_bf16_f32: round to nearest even
}

// 16 bytes at p -> kElems floats
__device__ inline void unpack16(const float *p, float (&out)[4]) {
    const float4 v = *reinterpret_cast<const float4 *>(p);
    out[0] = v.x;
    out[1] = v.y;
    out[2] = v.z;
    out[3] = v.w;
}
__device__ inline void unpack16(const bf16_t *p, float (&out)[8]) {
    const uint4 v = *reinterpret_cast<const uint4 *>(p);
    out[0] = __uint_as_float(v.x << 16);
    out[1] = __uint_as_float(v.x & 0xffff0000u);
    out[2] = __uint_as_float(v.y << 16);
    out[3] = __uint_as_float(v.y & 0xffff0000u);
    out[4] = __uint_as_float(v.z << 16);
    out[5] = __uint_as_float(v.z & 0xffff0000u);
    out[6] = __uint_as_float(v.w << 16);
    out[7] = __uint_as_float(v.w & 0xffff0000u);
}

// N floats -> N consecutive elements of T at p (p aligned to N * sizeof(T), N = 4 or 8)
template <int N>
__device__ inline void store_elems(float *p, const float (&v)[N]) {
#pragma unroll
    for (int i = 0; i < N; i += 4) *reinterpret_cast<float4 *>(p + i) = make_float4(v[i], v[i + 1], v[i + 2], v[i + 3]);
}
template <int N>
__device__ inline void store_elems(bf16_t *p, const float (&v)[N]) {
    typedef bf16_t bvec __attribute__((ext_vector_type(N)));
    bvec b;
#pragma unroll
    for (int i = 0; i < N; ++i) b[i] = (bf16_t)v[i];
    *reinterpret_cast<bvec *>(p) = b;
}

}  // namespace gcn

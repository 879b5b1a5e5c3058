// A float32 value as the exact sum of three bfloat16 values: the encoding with its low 16 bits cleared, the same
// of what is left after subtracting that, and the rest (8 + 8 + 8 significand bits).  Products of such planes on
// the bfloat16 matrix instruction, accumulated in float32, stand in for float32 products: the six plane pairs
// (i, j) with i + j <= 2 leave out terms below 2^-23 of |a| |b|.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace gcn {

// two bfloat16 (the upper halves of two float32 encodings) in one word: a in the low half, b in the high half
__device__ inline uint32_t pack_upper(uint32_t a, uint32_t b) {
    return __builtin_amdgcn_perm(b, a, 0x07060302u);   // bytes 2, 3 of a below bytes 2, 3 of b: one instruction
}

// Eight float32 encodings x[0..8) (consecutive rows of one column) -> `planes` operands of eight bfloat16 each:
// plane 0 the values with the low 16 bits cleared, plane 1 the same of what is left, plane 2 the rest (exact).
template <int PLANES>
__device__ inline void split_column(const uint32_t (&x)[8], uint4 (&out)[PLANES]) {
    uint32_t hi[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) hi[q] = pack_upper(x[2 * q], x[2 * q + 1]);
    out[0] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
    if (PLANES > 1) {
        uint32_t r1[8], r2[8], mid[4], lo[4];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            r1[i] = __float_as_uint(__uint_as_float(x[i]) - __uint_as_float(x[i] & 0xffff0000u));
            r2[i] = __float_as_uint(__uint_as_float(r1[i]) - __uint_as_float(r1[i] & 0xffff0000u));
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            mid[q] = pack_upper(r1[2 * q], r1[2 * q + 1]);
            lo[q] = pack_upper(r2[2 * q], r2[2 * q + 1]);
        }
        out[1] = make_uint4(mid[0], mid[1], mid[2], mid[3]);
        out[PLANES - 1] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    }
}

}  // namespace gcn

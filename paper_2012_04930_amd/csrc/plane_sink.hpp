// Epilogue helper of the dense products whose output is the next aggregation's input: besides the float32 rows
// the gather kernel reads, the same values go out as the three bfloat16 planes the tile product reads
// (tiles.hip, planes[p][ct][kg][c]: one 16-byte unit = plane p of rows 32 ct + 8 kg + 0..7 of column c), which
// saves that product a pass over the matrix.
#pragma once

#include "bf16_split.hpp"
#include "common.hpp"

namespace gcn {

// x[v], v = 0..15: the finished values of rows row0 + 8 (v / 4) + 4 h + v % 4 of column `col` (the accumulator
// layout of the 32 x 32 matrix instructions; row0 a multiple of 32), zero where the matrix has no such element.
// A lane holds four consecutive rows of each octet, i.e. one 8-byte half of a unit; the halves of lanes l and
// l + 32 are neighbours and the units of consecutive columns are consecutive, so a wave's store is 512 contiguous bytes.
__device__ inline void sink_store(const PlaneSink &s, int64_t row0, int col, int h, const float (&x)[16]) {
    const int64_t ct = row0 >> 5;
    if (col >= s.ld || ct >= s.n_ct) return;
    const size_t plane_units = (size_t)s.n_ct * 4 * s.ld;
    uint4 *planes = static_cast<uint4 *>(s.planes);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        uint32_t e[4], r1[4], r2[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            e[i] = __float_as_uint(x[4 * q + i]);
            r1[i] = __float_as_uint(x[4 * q + i] - __uint_as_float(e[i] & 0xffff0000u));
            r2[i] = __float_as_uint(__uint_as_float(r1[i]) - __uint_as_float(r1[i] & 0xffff0000u));
        }
        uint4 *unit = planes + ((size_t)ct * 4 + q) * s.ld + col;
        reinterpret_cast<uint2 *>(unit)[h] = make_uint2(pack_upper(e[0], e[1]), pack_upper(e[2], e[3]));
        reinterpret_cast<uint2 *>(unit + plane_units)[h] = make_uint2(pack_upper(r1[0], r1[1]), pack_upper(r1[2], r1[3]));
        reinterpret_cast<uint2 *>(unit + 2 * plane_units)[h] =
            make_uint2(pack_upper(r2[0], r2[1]), pack_upper(r2[2], r2[3]));
    }
}

}  // namespace gcn

// Epilogue helper of the dense products whose output is the next aggregation's input: besides the float32 rows
// the gather kernel reads, the same values go out in the order the tile product reads them (tiles.hip: a unit =
// rows 32 ct + 8 kg + 0..7 of column c as two 16-byte halves, units[((ct * 4 + kg) * 2 + half) * ld + c]), which
// saves that product a pass over the matrix.
#pragma once

#include "common.hpp"

namespace gcn {

// x[v], v = 0..15: the finished values of rows row0 + 8 (v / 4) + 4 h + v % 4 of column `col` (the accumulator
// layout of the 32 x 32 matrix instructions; row0 a multiple of 32), zero where the matrix has no such element.
// A lane holds four consecutive rows of each octet, i.e. exactly one half of a unit, and the halves of consecutive
// columns are consecutive: a wave's store is two runs of 512 contiguous bytes.
__device__ inline void sink_store(const PlaneSink &s, int64_t row0, int col, int h, const float (&x)[16]) {
    const int64_t ct = row0 >> 5;
    if (col >= s.ld || ct >= s.n_ct) return;
    uint4 *units = static_cast<uint4 *>(s.planes);
#pragma unroll
    for (int q = 0; q < 4; ++q)
        units[(((size_t)ct * 4 + q) * 2 + h) * s.ld + col] =
            make_uint4(__float_as_uint(x[4 * q]), __float_as_uint(x[4 * q + 1]), __float_as_uint(x[4 * q + 2]),
                       __float_as_uint(x[4 * q + 3]));
}

}  // namespace gcn

// Ceiling kernels: what the two units that the aggregation of Section 4.1's layer rule leans on deliver at
// best on this chip, measured in the same process as the kernels that are compared with them.
//   k_ceiling_gather     row gathers with the access shape of the aggregation kernels (a lane group per 16-byte-
//                        per-lane row, four loads in flight per lane, float32 adds), with the rows of each XCD's
//                        waves confined to one eighth of the table (every gather an L2 hit) or spread over all of it
//   k_ceiling_mfma_bf16  nothing but independent v_mfma_f32_32x32x16_bf16, the instruction of the tile product
#include "common.hpp"
#include "dtypes.hpp"
#include "epilogue.hpp"

namespace gcn {

namespace {

constexpr int kThreads = 256;

// LPR lanes per row (row_floats = 4 * LPR), GPW = 64 / LPR rows per load instruction.
template <int LPR>
__global__ __launch_bounds__(kThreads) void k_ceiling_gather(const float *__restrict__ table, uint32_t rows_per_part,
                                                             int n_parts, int row_floats, int64_t waves, int per_wave,
                                                             float *__restrict__ out) {
    constexpr int GPW = 64 / LPR, U = 4;
    const int lane = threadIdx.x & 63;
    const int grp = lane / LPR, sub = lane % LPR;
    const int64_t wave = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (wave >= waves) return;
    // the part of the table this wave's XCD reads from (n_parts = 1: the whole table)
    const uint32_t part = n_parts > 1 ? (uint32_t)(blockIdx.x % kXcds) : 0u;
    const uint32_t first_row = part * rows_per_part;
    const uint32_t row_bytes = (uint32_t)row_floats * 4u;
    const uint32_t lane_bytes = (uint32_t)sub * 16u;
    float acc0[4] = {0.f, 0.f, 0.f, 0.f}, acc1[4] = {0.f, 0.f, 0.f, 0.f};
    const uint64_t key = mix64((uint64_t)wave * 0x9E3779B97F4A7C15ull);
    for (int e = 0; e < per_wave; e += GPW * U) {
        float v[U][4];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            // one multiply-shift per row: the top bits of a 64-bit hash scaled to the part's row count
            const uint64_t hsh = mix64(key + (uint64_t)(e + u * GPW + grp));
            const uint32_t r = first_row + (uint32_t)(((hsh >> 32) * (uint64_t)rows_per_part) >> 32);
            const float4 q = *reinterpret_cast<const float4 *>(reinterpret_cast<const char *>(table) +
                                                               (size_t)r * row_bytes + lane_bytes);
            v[u][0] = q.x;
            v[u][1] = q.y;
            v[u][2] = q.z;
            v[u][3] = q.w;
        }
#pragma unroll
        for (int u = 0; u < U; u += 2)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc0[i] += v[u][i];
                acc1[i] += v[u + 1][i];
            }
    }
    float a[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = acc0[i] + acc1[i];
#pragma unroll
        for (int d = LPR; d < 64; d <<= 1) a[i] += __shfl_xor(a[i], d, 64);
    }
    if (grp == 0) *reinterpret_cast<float4 *>(out + wave * row_floats + sub * 4) = make_float4(a[0], a[1], a[2], a[3]);
}

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));

__global__ __launch_bounds__(kThreads) void k_ceiling_mfma_bf16(int64_t waves, int per_wave, float *__restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (wave >= waves) return;
    union {
        uint32_t u[4];
        bf16x8 v;
    } a, b;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a.u[i] = (lane & (1 << i)) ? 0x3F803F80u : 0x3F800000u;   // ones and zeros
        b.u[i] = 0x3C003C00u + (uint32_t)lane;                    // small finite values
    }
    f32x16 acc[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[k][v] = 0.0f;
    for (int i = 0; i < per_wave; ++i) {
#pragma unroll
        for (int k = 0; k < 4; ++k) acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, b.v, acc[k], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[k][v];
    out[wave * 64 + lane] = s;
}

}  // namespace

int ceiling_gather(const float *table, int64_t rows, int row_floats, int64_t waves, int per_wave, int spread, float *out,
                   hipStream_t st) {
    if (!table || !out || rows < 8 || rows > 0x7fffffff || row_floats < 4 || row_floats > 256 || row_floats % 4 != 0 ||
        waves < 1 || per_wave < 1 || (uint64_t)rows * (uint64_t)row_floats * 4ull > 0xffffffffull) {
        set_error("gcn_ceiling_gather: bad argument (8 <= rows, row_floats a multiple of 4 up to 256, table below 4 GiB)");
        return GCN_EINVAL;
    }
    const int n_parts = spread ? 1 : kXcds;
    const uint32_t rows_per_part = (uint32_t)(rows / n_parts);
    const unsigned grid = (unsigned)((waves + kThreads / 64 - 1) / (kThreads / 64));
    const int lpr = row_floats / 4;
#define GCN_CEIL(LPR)                                                                                                  \
    k_ceiling_gather<LPR><<<dim3(grid), dim3(kThreads), 0, st>>>(table, rows_per_part, n_parts, row_floats, waves,     \
                                                                 per_wave, out)
    if (lpr > 32) GCN_CEIL(64);
    else if (lpr > 16) GCN_CEIL(32);
    else if (lpr > 8) GCN_CEIL(16);
    else if (lpr > 4) GCN_CEIL(8);
    else GCN_CEIL(4);
#undef GCN_CEIL
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int ceiling_mfma_bf16(int64_t waves, int per_wave, float *out, hipStream_t st) {
    if (!out || waves < 1 || per_wave < 1) {
        set_error("gcn_ceiling_mfma_bf16: bad argument");
        return GCN_EINVAL;
    }
    k_ceiling_mfma_bf16<<<dim3((unsigned)((waves + kThreads / 64 - 1) / (kThreads / 64))), dim3(kThreads), 0, st>>>(
        waves, per_wave, out);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

}  // namespace gcn

extern "C" int gcn_ceiling_gather(const float *table, int64_t rows, int32_t row_floats, int64_t waves, int32_t per_wave,
                                  int spread, float *out, void *stream) {
    return gcn::ceiling_gather(table, rows, row_floats, waves, per_wave, spread, out, (hipStream_t)stream);
}

extern "C" int gcn_ceiling_mfma_bf16(int64_t waves, int32_t per_wave, float *out, void *stream) {
    return gcn::ceiling_mfma_bf16(waves, per_wave, out, (hipStream_t)stream);
}

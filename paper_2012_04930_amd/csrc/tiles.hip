// Dense panels of the adjacency pattern, for the aggregation  Z = A_hat T  of Section 4.1's layer rule.
//
// A partition of a community-structured graph (the paper's partitions come from a min-cut partitioner,
// Section 3; its Reddit workload averages about 490 neighbours per vertex, Table 1) holds blocks of the
// adjacency pattern that are a third full, and the vertices that stand in for the other partitions
// (Section 3.1) are adjacent to a few percent of all local vertices.  For such a block the gather form of
// the product reads one input row per stored entry, hundreds of times the same few rows, and is bound by
// cache throughput.  As a product of a zero/one block with a slab of the input it reads each input row once
// per 128 output rows and runs on the matrix cores.
//
// At graph creation the pattern is cut into aligned panels of kTileRows = 128 rows by 32 columns.  Panels with
// at least `min_entries` stored entries become "dense tiles": a column-tile index and 128 words of 32 bits
// (word r = which of the 32 columns row r holds).  Everything else stays in a residual CSR with the usual
// schedules.  An aggregation is then two parts: k_tiles writes the plain sums over the dense tiles of every
// row, and the gather kernels add the residual entries and finish (scaling by d_i^-1/2, activation).  Graphs
// without such blocks (selected tiles hold under a quarter of the entries) keep the single-launch gather form.
//
// The product itself: a float32 input row is split exactly into three bfloat16 numbers, x = hi + mid + lo
// (8 + 8 + 8 significant bits: hi = x with the low 16 bits of its encoding cleared, mid likewise from x - hi, lo
// = the rest, which then has at most 8 significant bits; all three subtractions are exact).  Ones and zeros are
// exact in bfloat16 too, so three passes of v_mfma_f32_32x32x16_bf16 over the same accumulator add exactly
// the terms the float32 gather adds, in float32, in another order.  (Values below 2^-110 lose their last bits:
// bfloat16 has float32's exponent range but lo is 2^-16 times smaller.)  bfloat16 input rows need one pass.
// The input reaches k_tiles in the order the instruction reads its second operand ("units", see k_tile_planes);
// float32 units are split into the three planes in registers.  Who writes the units: the kernel that produces the
// aggregation's input, from its epilogue (plane_sink.hpp; the dense products and the loss kernel), or else the
// pass k_tile_planes.
#include <algorithm>
#include <vector>

#include "common.hpp"
#include "dtypes.hpp"
#include "bf16_split.hpp"

namespace gcn {

namespace {

constexpr int kThreads = 256;
constexpr int kChunk = 8192;   // column tiles counted per pass: 32 KB of LDS counters

inline unsigned blocks_for(int64_t items, int per_block) { return (unsigned)((items + per_block - 1) / per_block); }

// One workgroup per row block (kTileRows rows).  Counts the entries of every column tile (32 columns) in LDS, a
// chunk of column tiles at a time, and selects the panels with at least min_entries, in ascending column order.
//   WRITE = false: tile_cnt[rt] = number selected; totals[0] += entries in selected tiles
//   WRITE = true : tile_col / tile_rt filled from tile_ptr[rt] on
template <bool WRITE>
__global__ __launch_bounds__(kThreads) void k_tile_select(int64_t n, int64_t n_ct, const int64_t *__restrict__ rowptr,
                                                          const int32_t *__restrict__ col, int min_entries,
                                                          int32_t *__restrict__ tile_cnt,
                                                          const int64_t *__restrict__ tile_ptr,
                                                          int32_t *__restrict__ tile_col,
                                                          int32_t *__restrict__ tile_rt,
                                                          unsigned long long *__restrict__ totals) {
    __shared__ uint32_t cnt[kChunk];
    __shared__ int wave_total[kThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t rt = blockIdx.x;
    const int64_t r0 = rt * kTileRows;
    const int64_t r1 = r0 + kTileRows < n ? r0 + kTileRows : n;
    const int64_t e0 = rowptr[r0], e1 = rowptr[r1];
    int running = 0;
    unsigned long long my_entries = 0;
    const int64_t out0 = WRITE ? tile_ptr[rt] : 0;
    for (int64_t cb = 0; cb < n_ct; cb += kChunk) {
        const int m = (int)(n_ct - cb < kChunk ? n_ct - cb : kChunk);
        for (int i = tid; i < m; i += kThreads) cnt[i] = 0;
        __syncthreads();
        for (int64_t e = e0 + tid; e < e1; e += kThreads) {
            const int64_t ct = (int64_t)(col[e] >> 5) - cb;
            if (ct >= 0 && ct < m) atomicAdd(&cnt[ct], 1u);
        }
        __syncthreads();
        for (int base = 0; base < m; base += kThreads) {
            const int i = base + tid;
            const uint32_t c = i < m ? cnt[i] : 0u;
            const bool sel = c >= (uint32_t)min_entries;
            const unsigned long long b = __ballot(sel);
            if (lane == 0) wave_total[wave] = __popcll(b);
            __syncthreads();
            int off = __popcll(b & ((1ull << lane) - 1ull));
            int total = 0;
#pragma unroll
            for (int w = 0; w < kThreads / 64; ++w) {
                if (w < wave) off += wave_total[w];
                total += wave_total[w];
            }
            if (sel) {
                my_entries += c;
                if (WRITE) {
                    tile_col[out0 + running + off] = (int32_t)(cb + i);
                    tile_rt[out0 + running + off] = (int32_t)rt;
                }
            }
            running += total;
            __syncthreads();
        }
    }
    if (!WRITE) {
        if (tid == 0) tile_cnt[rt] = running;
#pragma unroll
        for (int d = 32; d > 0; d >>= 1) my_entries += __shfl_xor(my_entries, d, 64);
        if (lane == 0 && my_entries) atomicAdd(totals, my_entries);
    }
}

// true when column tile ct is among the (ascending) dense tiles tile_col[lo .. end)
__device__ inline bool tile_is_dense(const int32_t *__restrict__ tile_col, int64_t lo, int64_t end, int ct) {
    int64_t hi = end;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (tile_col[mid] < ct) lo = mid + 1; else hi = mid;
    }
    return lo < end && tile_col[lo] == ct;
}

// One thread per (dense tile, row of the tile): the 32-bit word of columns that the row holds inside the tile
// (zero for rows past the end of the matrix).
__global__ void k_tile_bits(int64_t n, int64_t n_tiles, const int64_t *__restrict__ rowptr,
                            const int32_t *__restrict__ col, const int32_t *__restrict__ tile_col,
                            const int32_t *__restrict__ tile_rt, uint32_t *__restrict__ bits) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_tiles * kTileRows) return;
    const int64_t ti = i / kTileRows;
    const int64_t r = (int64_t)tile_rt[ti] * kTileRows + (i % kTileRows);
    uint32_t word = 0;
    if (r < n) {
        const int c0 = tile_col[ti] * 32;
        const int64_t end = rowptr[r + 1];
        int64_t lo = rowptr[r], hi = end;
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            if (col[mid] < c0) lo = mid + 1; else hi = mid;
        }
        for (; lo < end; ++lo) {
            const int c = col[lo];
            if (c >= c0 + 32) break;
            word |= 1u << (c - c0);
        }
    }
    bits[i] = word;
}

// One wave per row: the entries outside the dense tiles of the row's block, in their order.
//   WRITE = false: res_deg[r] = how many;  WRITE = true: res_col filled from res_rowptr[r] on
template <bool WRITE>
__global__ __launch_bounds__(kThreads) void k_residual(int64_t n, const int64_t *__restrict__ rowptr,
                                                       const int32_t *__restrict__ col,
                                                       const int64_t *__restrict__ tile_ptr,
                                                       const int32_t *__restrict__ tile_col,
                                                       int32_t *__restrict__ res_deg,
                                                       const int64_t *__restrict__ res_rowptr,
                                                       int32_t *__restrict__ res_col) {
    const int64_t r = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (r >= n) return;
    const int lane = threadIdx.x & 63;
    const int64_t lo = tile_ptr[r / kTileRows], hi = tile_ptr[r / kTileRows + 1];
    const int64_t beg = rowptr[r], end = rowptr[r + 1];
    const int64_t out0 = WRITE ? res_rowptr[r] : 0;
    int count = 0;
    for (int64_t e0 = beg; e0 < end; e0 += 64) {
        const int64_t e = e0 + lane;
        int c = 0;
        bool keep = false;
        if (e < end) {
            c = col[e];
            keep = !tile_is_dense(tile_col, lo, hi, c >> 5);
        }
        const unsigned long long b = __ballot(keep);
        if (WRITE && keep) res_col[out0 + count + __popcll(b & ((1ull << lane) - 1ull))] = c;
        count += __popcll(b);
    }
    if (!WRITE && lane == 0) res_deg[r] = count;
}

// ------------------------------------------------------------------------------------------------ the product
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));

template <typename TIn>
struct Planes;
template <>
struct Planes<float> {
    static constexpr int kCount = 3;
};
template <>
struct Planes<bf16_t> {
    static constexpr int kCount = 1;
};

// Two consecutive elements of a row, as float32 encodings.
__device__ inline void load_pair(const float *p, uint32_t (&v)[2]) {
    const uint2 q = *reinterpret_cast<const uint2 *>(p);
    v[0] = q.x;
    v[1] = q.y;
}
__device__ inline void load_pair(const bf16_t *p, uint32_t (&v)[2]) {
    const uint32_t q = *reinterpret_cast<const uint32_t *>(p);
    v[0] = q << 16;
    v[1] = q & 0xffff0000u;
}

// ---- step 1: the input in the order the matrix instruction reads its second operand.
// A unit holds t[32 ct + 8 kg + 0 .. 7, c], the eight consecutive-k values of one k-octet of one column, units
// ordered (ct, kg, c) major to minor, c < ld.  bfloat16 input: 16 bytes per unit, units[(ct * 4 + kg) * ld + c].
// float32 input: the eight float32 values as two 16-byte halves (rows 0 .. 3 and 4 .. 7 of the octet),
// units[((ct * 4 + kg) * 2 + half) * ld + c]; the product splits them into three bfloat16 planes in registers (the
// same 4 bytes per element through the caches as the matrix itself, where three stored planes would be 6).
// Rows at or past n and columns at or past `cols` are zero (ld, the units' own leading dimension, is cols rounded
// up to whole blocks of 32).  One thread per (ct, kg, pair of columns): eight rows of two columns in, two units out.
template <typename TIn>
__global__ __launch_bounds__(kThreads) void k_tile_planes(const TIn *__restrict__ t, int ld_t, int64_t n, int n_ct,
                                                          int cols, int ld, uint4 *__restrict__ planes) {
    constexpr int P = Planes<TIn>::kCount;
    const int pairs = ld / 2;
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= (int64_t)n_ct * 4 * pairs) return;
    const int c2 = (int)(i % pairs);
    const int kg = (int)((i / pairs) % 4);
    const int64_t ct = i / ((int64_t)pairs * 4);
    const int64_t row0 = ct * 32 + kg * 8;
    uint32_t r[8][2];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        r[k][0] = r[k][1] = 0u;
        if (row0 + k < n && 2 * c2 < cols) load_pair(t + (row0 + k) * ld_t + 2 * c2, r[k]);   // cols is even
    }
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        if (P == 1) {
            uint32_t x[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) x[k] = r[k][c];
            uint4 o[1];
            split_column<1>(x, o);
            planes[((size_t)ct * 4 + kg) * ld + 2 * c2 + c] = o[0];
        } else {
            uint4 *unit = planes + ((size_t)ct * 4 + kg) * 2 * ld + 2 * c2 + c;
            unit[0] = make_uint4(r[0][c], r[1][c], r[2][c], r[3][c]);
            unit[ld] = make_uint4(r[4][c], r[5][c], r[6][c], r[7][c]);
        }
    }
}

// ---- step 2: the product.  One workgroup (4 independent waves; LDS holds only a 128-byte table) per work item = a run of dense
// tiles of one row block (kTileRows output rows) and, with blockIdx.y, a span of 32 NBLK columns:
//   dst[rows of the block, the span] = sum over the run's tiles of  bits (kTileRows x 32, zero/one) x planes(ct).
// NBLK = 4: wave w takes column block w (32 columns) of all four row tiles (32 rows each) of the block; NBLK = 2:
// column block w % 2 of two row tiles; NBLK = 1: one row tile each.  Per tile and 16-deep k-step a wave loads one
// 16-byte unit per plane and lane straight from memory (lane l: column l % 32 of its block, k-octet l / 32),
// turns the bit words of its row tiles into bfloat16 ones and zeros through a 16-entry table, and issues one matrix
// instruction per row tile and plane, consecutive ones into different accumulators.  Loads run three tiles ahead
// in three register stages; no branch inside a step.
// Waves whose column block lies at or past `cols` leave at once.
struct TileItem {
    int32_t rb;      // row block
    int32_t first;   // index of the run's first dense tile
    int32_t count;   // tiles in the run (0: the block has none and its sums are zero)
    int32_t slot;    // -1: the sums go to the output rows; k >= 0: to block k of the partial-sum buffer
};

template <int P, int NBLK>
__global__ __launch_bounds__(kThreads) void k_tiles(const TileItem *__restrict__ items,
                                                    const int32_t *__restrict__ tile_col,
                                                    const uint32_t *__restrict__ bits, int64_t n, int n_ct,
                                                    const uint4 *__restrict__ planes, int ld, float *__restrict__ out,
                                                    int ld_out, float *__restrict__ partial, int cols) {
    constexpr int WM = 4 / NBLK;                   // waves stacked over the rows
    constexpr int SUB = kTileRows / 32 / WM;       // row tiles of 32 per wave
    static_assert(NBLK == 1 || NBLK == 2 || NBLK == 4, "32, 64 or 128 columns per workgroup");
    const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, l32 = lane & 31;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave % NBLK, wm = wave / NBLK;
    // entry e of the table: bit i of e -> bfloat16 one (0x3F80) or zero in element i, i = 0..3
    __shared__ uint2 lut[16];
    if (tid < 16) {
        const uint32_t e = (uint32_t)tid;
        lut[tid] = make_uint2(((e & 1u) ? 0x3F80u : 0u) | ((e & 2u) ? 0x3F800000u : 0u),
                              ((e & 4u) ? 0x3F80u : 0u) | ((e & 8u) ? 0x3F800000u : 0u));
    }
    __syncthreads();   // the only barrier: before any wave leaves
    // workgroup b runs on XCD b mod 8 and takes place b / 8 of that XCD's sub-list (gridDim.x = 8 x its length)
    const TileItem item = items[(blockIdx.x % kXcds) * (gridDim.x / kXcds) + blockIdx.x / kXcds];
    if (item.rb < 0) return;                       // an unused place
    const int col = (blockIdx.y * NBLK + wn) * 32 + l32;
    if (col - l32 >= cols) return;                 // the whole wave: nothing of its block is inside the matrix
    const int64_t first = item.first;
    const int count = item.count;
    // pieces of 16 bytes per unit: one (bfloat16 input) or two (float32 input, split below)
    constexpr int Q = P == 1 ? 1 : 2;
    // piece q of k-step s for this lane inside tile ct:  (ct * 4 + 2 s + h) * Q * ld + q * ld + col
    const uint32_t lane_unit = (uint32_t)(h * Q * ld + col);   // col < ld: the units cover whole blocks of 32 columns

    struct Stage {
        uint4 b[2][Q];
        uint32_t w[SUB];
    };
    // Loads of tile i (clamped into the run, so they are always valid).  The tile's column index was fetched by the
    // fill before (ct_next), so no load here waits for another.
    int ct_next = tile_col[first];
    auto fill = [&](int i, Stage &st) {
        const int64_t ti = first + (i < count ? i : count - 1);
        const int ct = ct_next;
        ct_next = tile_col[first + (i + 1 < count ? i + 1 : count - 1)];
        const uint4 *base = planes + (size_t)ct * 4 * Q * ld;   // wave-uniform
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int q = 0; q < Q; ++q) st.b[s][q] = base[(size_t)(2 * s * Q + q) * ld + lane_unit];
#pragma unroll
        for (int u = 0; u < SUB; ++u) st.w[u] = bits[ti * kTileRows + (wm * SUB + u) * 32 + l32];
    };

    f32x16 acc[SUB];
#pragma unroll
    for (int u = 0; u < SUB; ++u)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[u][v] = 0.0f;

    if (count > 0) {
        Stage s0, s1, s2;
        // Bits to operands: four bits pick one of the 16 entries of a table in LDS, each four bfloat16 ones and
        // zeros (8 bytes; the 16 entries lie in 32 different banks and lanes that read the same entry share it, so
        // the reads never conflict).  Two table reads per row tile and k-step instead of ten vector instructions,
        // which on this chip do not run in the shadow of the matrix instructions.
        auto operand = [&](uint32_t w, int sh) {
            union {
                uint2 half[2];
                bf16x8 v;
            } r;
            r.half[0] = lut[(w >> sh) & 15u];
            r.half[1] = lut[(w >> (sh + 4)) & 15u];
            return r.v;
        };
        auto step = [&](int i, Stage &st) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                bf16x8 a[SUB];
#pragma unroll
                for (int u = 0; u < SUB; ++u) a[u] = operand(st.w[u], 16 * s + 8 * h);
                uint4 plane[P];
                if (P == 1) {
                    plane[0] = st.b[s][0];
                } else {
                    const uint32_t x[8] = {st.b[s][0].x,     st.b[s][0].y,     st.b[s][0].z,     st.b[s][0].w,
                                           st.b[s][Q - 1].x, st.b[s][Q - 1].y, st.b[s][Q - 1].z, st.b[s][Q - 1].w};
                    split_column<P>(x, plane);
                }
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    union {
                        uint4 q;
                        bf16x8 v;
                    } b;
                    b.q = plane[p];
#pragma unroll
                    for (int u = 0; u < SUB; ++u)
                        acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u], b.v, acc[u], 0, 0, 0);
                }
            }
            fill(i + 3, st);   // the stage's registers have been read: its next tile's loads go out now
        };
        fill(0, s0);
        fill(1, s1);
        fill(2, s2);
        for (int i = 0; i < count; i += 3) {
            step(i, s0);
            if (i + 1 < count) step(i + 1, s1);
            if (i + 2 < count) step(i + 2, s2);
        }
    }
    // accumulator element v of lane l: row 8 (v / 4) + 4 (l / 32) + v % 4 of the row tile, column l % 32 of the block
    if (col >= cols) return;
    // partial sums are kept compact: blocks of kTileRows x cols floats
    float *dst = item.slot < 0 ? out + (int64_t)item.rb * kTileRows * ld_out
                               : partial + (int64_t)item.slot * kTileRows * cols;
    const int ld_dst = item.slot < 0 ? ld_out : cols;
    const int64_t rows_left = n - (int64_t)item.rb * kTileRows;   // rows of this block inside the matrix
#pragma unroll
    for (int u = 0; u < SUB; ++u)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = (wm * SUB + u) * 32 + 8 * (v / 4) + 4 * h + (v % 4);
            if (row < rows_left) dst[(int64_t)row * ld_dst + col] = acc[u][v];
        }
}

// Row blocks whose tiles were cut into several runs: the runs' partial sums are added to the block's output
// rows in run order.  One thread per (fold entry, row of the block, four columns).
struct TileFold {
    int32_t rb, slot0, slots, pad;
};
__global__ __launch_bounds__(kThreads) void k_tiles_fold(const TileFold *__restrict__ folds, int n_folds, int64_t n,
                                                         float *__restrict__ out, int ld_out,
                                                         const float *__restrict__ partial, int cols) {
    const int quads = cols / 4;
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= (int64_t)n_folds * kTileRows * quads) return;
    const int c0 = (int)(i % quads) * 4;
    const int row = (int)((i / quads) % kTileRows);
    const TileFold f = folds[i / ((int64_t)quads * kTileRows)];
    const int64_t r = (int64_t)f.rb * kTileRows + row;
    if (r >= n) return;
    float4 o = *reinterpret_cast<const float4 *>(out + r * ld_out + c0);
#pragma unroll 8
    for (int k = 0; k < f.slots; ++k) {
        const float4 q =
            *reinterpret_cast<const float4 *>(partial + ((int64_t)(f.slot0 + k) * kTileRows + row) * cols + c0);
        o.x += q.x;
        o.y += q.y;
        o.z += q.z;
        o.w += q.w;
    }
    *reinterpret_cast<float4 *>(out + r * ld_out + c0) = o;
}

}  // namespace

size_t tiles_capacity(int64_t entries) { return (size_t)(entries / kTileMinEntriesFloor) + 1; }
size_t tiles_item_capacity(int64_t n_rb, int64_t tile_capacity) {
    return (size_t)kXcds * (size_t)(2 * n_rb + tile_capacity / kTileChunkMin + 16);   // eight padded sub-lists
}

int tiles_select(int64_t n, const int64_t *rowptr, const int32_t *col, int min_entries, TileBuffers &tb,
                 int64_t *blocksum, hipStream_t st) {
    if (min_entries < kTileMinEntriesFloor || min_entries > kTileRows * 32) {
        set_error("dense tiles: the entry threshold must lie in [%d, %d]", kTileMinEntriesFloor, kTileRows * 32);
        return GCN_EINVAL;
    }
    const int64_t n_ct = (n + 31) / 32;
    int rc = fill_zero(tb.totals, sizeof(unsigned long long), st);
    if (rc) return rc;
    k_tile_select<false><<<dim3((unsigned)tb.n_rb), dim3(kThreads), 0, st>>>(n, n_ct, rowptr, col, min_entries,
                                                                              tb.tile_cnt, nullptr, nullptr, nullptr,
                                                                              tb.totals);
    GCN_LAUNCH_CHECK();
    rc = exclusive_scan_i32(tb.n_rb, tb.tile_cnt, tb.tile_ptr, blocksum, st);
    if (rc) return rc;
    k_tile_select<true><<<dim3((unsigned)tb.n_rb), dim3(kThreads), 0, st>>>(n, n_ct, rowptr, col, min_entries,
                                                                             nullptr, tb.tile_ptr, tb.tile_col,
                                                                             tb.tile_rt, nullptr);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int tiles_build(int64_t n, const int64_t *rowptr, const int32_t *col, int64_t n_tiles, TileBuffers &tb,
                PrepBuffers &res, hipStream_t st) {
    if (n_tiles > 0) {
        k_tile_bits<<<dim3(blocks_for(n_tiles * kTileRows, kThreads)), dim3(kThreads), 0, st>>>(
            n, n_tiles, rowptr, col, tb.tile_col, tb.tile_rt, tb.bits);
        GCN_LAUNCH_CHECK();
    }
    k_residual<false><<<dim3(blocks_for(n, kThreads / 64)), dim3(kThreads), 0, st>>>(n, rowptr, col, tb.tile_ptr,
                                                                                      tb.tile_col, res.deg, nullptr,
                                                                                      nullptr);
    GCN_LAUNCH_CHECK();
    int rc = exclusive_scan_i32(n, res.deg, res.rowptr, res.blocksum, st);
    if (rc) return rc;
    k_residual<true><<<dim3(blocks_for(n, kThreads / 64)), dim3(kThreads), 0, st>>>(n, rowptr, col, tb.tile_ptr,
                                                                                     tb.tile_col, nullptr, res.rowptr,
                                                                                     res.col);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

// The work items of the product, from the number of dense tiles of every row block (tile_ptr on the host).
// The chip holds kSlots workgroups of k_tiles at a time and hands a freed place to the next workgroup in launch
// order, so the list is: first one item per ordinary row block (a block with about the average number of tiles per
// place, or fewer), then the tiles of the blocks that hold far more, cut into short runs that fill whatever places
// are free until all end together.  The first run of such a block writes the output rows, the others partial sums
// that k_tiles_fold adds in run order.
// Layout: workgroup b runs on XCD b mod 8 (each XCD has its own L2), so the list is eight sub-lists,
// items[x * per_xcd + i] for workgroup 8 i + x.  Each sub-list is a contiguous eighth (by tile count) of the ordinary
// blocks in row order (the blocks of one community read the same input rows and meet in one L2) followed by a
// contiguous eighth of the runs, ordered by position inside their block (runs at the same position read the same
// input rows).  Unused places hold rb = -1.
int tiles_plan(const std::vector<int64_t> &tile_ptr, TileBuffers &tb, hipStream_t st) {
    const int64_t n_rb = (int64_t)tile_ptr.size() - 1;
    const int64_t total = tile_ptr[n_rb];
    int64_t kSlots = tunable("tile_slots", 768);   // workgroups of k_tiles the chip is taken to hold at a time
    if (kSlots < 256) kSlots = 256;
    int64_t run = (total + kSlots - 1) / kSlots;
    const int64_t run_min = tunable("tile_run_min", kTileRunMin);
    if (run < run_min) run = run_min;
    // (an item of hundreds of tiles ends late: the full Reddit shape, 270,513 tiles, 352 per place: 137.3 epochs/s,
    // with at most 128 to an item 139.0)
    const int64_t run_max = tunable("tile_run_max", 128);
    if (run > run_max && run_max >= run_min) run = run_max;
    int64_t chunk = tunable("tile_chunk", 0);
    if (chunk <= 0) chunk = run * 3 / 4;   // (benchmark partition, epoch: run / 2 1.125 ms, 3/4 1.107, 1 1.114, 3/2 1.121)
    if (chunk < kTileChunkMin) chunk = kTileChunkMin;
    std::vector<TileItem> whole, cut;
    std::vector<int> cut_pos;   // position of a run inside its block
    std::vector<TileFold> folds;
    int32_t slots = 0;
    for (int64_t rb = 0; rb < n_rb; ++rb) {
        const int64_t first = tile_ptr[rb], cnt = tile_ptr[rb + 1] - first;
        if (cnt * 2 <= run * 3) {
            whole.push_back({(int32_t)rb, (int32_t)first, (int32_t)cnt, -1});
            continue;
        }
        const int64_t parts = (cnt + chunk - 1) / chunk;
        folds.push_back({(int32_t)rb, slots, (int32_t)(parts - 1), 0});
        for (int64_t k = 0; k < parts; ++k) {
            const int64_t b = first + cnt * k / parts, e = first + cnt * (k + 1) / parts;
            cut.push_back({(int32_t)rb, (int32_t)b, (int32_t)(e - b), k == 0 ? -1 : slots++});
            cut_pos.push_back((int)k);
        }
    }
    {
        std::vector<size_t> order(cut.size());
        for (size_t i = 0; i < order.size(); ++i) order[i] = i;
        std::stable_sort(order.begin(), order.end(), [&](size_t x, size_t y) { return cut_pos[x] < cut_pos[y]; });
        std::vector<TileItem> sorted;
        sorted.reserve(cut.size());
        for (size_t i : order) sorted.push_back(cut[i]);
        cut.swap(sorted);
    }
    // eight contiguous pieces of about equal numbers of tiles (an item counts as at least one)
    auto eighths = [](const std::vector<TileItem> &seq, std::vector<size_t> &start) {
        int64_t weight = 0;
        for (const TileItem &it : seq) weight += it.count > 0 ? it.count : 1;
        start.assign(kXcds + 1, seq.size());
        start[0] = 0;
        int64_t done = 0;
        size_t i = 0;
        for (int x = 1; x < kXcds; ++x) {
            const int64_t want = weight * x / kXcds;
            while (i < seq.size() && done < want) {
                done += seq[i].count > 0 ? seq[i].count : 1;
                ++i;
            }
            start[x] = i;
        }
    };
    std::vector<size_t> ws, cs;
    eighths(whole, ws);
    eighths(cut, cs);
    size_t per_xcd = 0;
    for (int x = 0; x < kXcds; ++x) per_xcd = std::max(per_xcd, (ws[x + 1] - ws[x]) + (cs[x + 1] - cs[x]));
    std::vector<TileItem> items(per_xcd * kXcds, TileItem{-1, 0, 0, -1});
    for (int x = 0; x < kXcds; ++x) {
        size_t at = x * per_xcd;
        for (size_t i = ws[x]; i < ws[x + 1]; ++i) items[at++] = whole[i];
        for (size_t i = cs[x]; i < cs[x + 1]; ++i) items[at++] = cut[i];
    }
    if (items.size() > tb.item_capacity || folds.size() > (size_t)n_rb || total > 0x7fffffff) {
        set_error("dense tiles: %zu work items exceed the capacity %zu", items.size(), tb.item_capacity);
        return GCN_EINVAL;
    }
    static_assert(sizeof(TileItem) == 16 && sizeof(TileFold) == 16, "four 32-bit words each");
    tb.n_items = (int32_t)items.size();
    tb.n_folds = (int32_t)folds.size();
    tb.n_slots = slots;
    if (!items.empty())
        GCN_HIP(hipMemcpyAsync(tb.items, items.data(), items.size() * sizeof(TileItem), hipMemcpyHostToDevice, st));
    if (!folds.empty())
        GCN_HIP(hipMemcpyAsync(tb.folds, folds.data(), folds.size() * sizeof(TileFold), hipMemcpyHostToDevice, st));
    GCN_HIP(hipStreamSynchronize(st));   // the vectors go out of scope
    return GCN_OK;
}

size_t tiles_plane_bytes(int64_t n, int cols, int dtype) {
    const size_t n_ct = (size_t)((n + 31) / 32);
    return (size_t)(dtype == GCN_BF16 ? 1 : 2) * n_ct * 4 * (size_t)round_up(cols, 32) * 16;
}

PlaneSink tiles_plane_sink(const SpmmArgs &a) {
    if (!a.tile_ptr || !a.tile_planes || a.t_dtype != GCN_F32 || a.cols > 256 || tunable("fused_planes", 1) == 0)
        return PlaneSink{nullptr, 0, 0};
    return PlaneSink{a.tile_planes, (int)((a.n + 31) / 32), (int)round_up(a.cols, 32)};
}

// the input of aggregation `a` as the product's operand planes (nothing to do when its producer wrote them)
int tiles_planes(const SpmmArgs &a, hipStream_t st) {
    if (a.planes_ready) return GCN_OK;
    if (a.cols > 256 || !a.tile_planes) {
        set_error("dense tiles: at most 256 columns and a buffer for the operand planes");
        return GCN_EINVAL;
    }
    const int n_ct = (int)((a.n + 31) / 32);
    const int ld = (int)round_up(a.cols, 32);
    uint4 *planes = static_cast<uint4 *>(a.tile_planes);
    const int64_t threads = (int64_t)n_ct * 4 * (ld / 2);
    const int t_planes = timing_open(kTimePlanes, a.width, st);
    if (a.t_dtype == GCN_BF16)
        k_tile_planes<bf16_t><<<dim3(blocks_for(threads, kThreads)), dim3(kThreads), 0, st>>>(
            static_cast<const bf16_t *>(a.t), a.ld_t, a.n, n_ct, a.cols, ld, planes);
    else
        k_tile_planes<float><<<dim3(blocks_for(threads, kThreads)), dim3(kThreads), 0, st>>>(
            static_cast<const float *>(a.t), a.ld_t, a.n, n_ct, a.cols, ld, planes);
    GCN_LAUNCH_CHECK();
    timing_close(t_planes, st);
    return GCN_OK;
}

int units_from_rows(const float *t, int ld_t, int64_t n, int cols, void *units, hipStream_t st) {
    if (n <= 0) return GCN_OK;
    if (cols <= 0 || cols % 2 != 0 || ld_t < cols) {
        set_error("units_from_rows: an even number of columns within the leading dimension (cols=%d ld=%d)", cols, ld_t);
        return GCN_EINVAL;
    }
    const int n_ct = (int)((n + 31) / 32);
    const int ld = (int)round_up(cols, 32);
    const int64_t threads = (int64_t)n_ct * 4 * (ld / 2);
    k_tile_planes<float><<<dim3(blocks_for(threads, kThreads)), dim3(kThreads), 0, st>>>(t, ld_t, n, n_ct, cols, ld,
                                                                                     static_cast<uint4 *>(units));
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

// (after tiles_planes, on a stream ordered behind it)
int tiles_launch(const SpmmArgs &a, float *dst, int ld_dst, hipStream_t st) {
    if (a.cols > 256 || a.n_items < 1 || (a.n_slots > 0 && !a.tile_partial) || !a.tile_planes) {
        set_error("dense tiles: at most 256 columns, a buffer for the operand planes, and one for partial sums when runs were cut");
        return GCN_EINVAL;
    }
    const int n_ct = (int)((a.n + 31) / 32);
    const int ld = (int)round_up(a.cols, 32);
    uint4 *planes = static_cast<uint4 *>(a.tile_planes);
    const int t_tiles = timing_open(kTimeTiles, a.width, st);
    const TileItem *items = reinterpret_cast<const TileItem *>(a.tile_items);
#define GCN_TILES(NBLK)                                                                                               \
    do {                                                                                                              \
        const dim3 grid((unsigned)a.n_items, (unsigned)((a.cols + 32 * NBLK - 1) / (32 * NBLK)));                     \
        if (a.t_dtype == GCN_BF16)                                                                                    \
            k_tiles<1, NBLK><<<grid, dim3(kThreads), 0, st>>>(items, a.tile_col, a.bits, a.n, n_ct, planes, ld, dst,  \
                                                              ld_dst, a.tile_partial, a.cols);                        \
        else                                                                                                          \
            k_tiles<3, NBLK><<<grid, dim3(kThreads), 0, st>>>(items, a.tile_col, a.bits, a.n, n_ct, planes, ld, dst,  \
                                                              ld_dst, a.tile_partial, a.cols);                        \
    } while (0)
    if (a.cols <= 32) GCN_TILES(1);
    else if (a.cols <= 64) GCN_TILES(2);
    else GCN_TILES(4);
#undef GCN_TILES
    GCN_LAUNCH_CHECK();
    if (a.n_folds > 0) {
        const int64_t fthreads = (int64_t)a.n_folds * kTileRows * (a.cols / 4);
        k_tiles_fold<<<dim3(blocks_for(fthreads, kThreads)), dim3(kThreads), 0, st>>>(
            reinterpret_cast<const TileFold *>(a.tile_folds), a.n_folds, a.n, dst, ld_dst, a.tile_partial, a.cols);
        GCN_LAUNCH_CHECK();
    }
    timing_close(t_tiles, st);
    return GCN_OK;
}

}  // namespace gcn

// Dense tiles of the adjacency pattern, for the aggregation  Z = A_hat T  of Section 4.1's layer rule.
//
// A partition of a community-structured graph (the paper's partitions come from a min-cut partitioner,
// Section 3; its Reddit workload averages about 490 neighbours per vertex, Table 1) holds blocks of the
// adjacency pattern that are a third full.  For such a block the gather form of the product reads a 512-byte
// input row per stored entry, hundreds of times the same few rows, and is bound by cache throughput; as a
// product of a 32 x 32 zero/one block with a 32 x w slab of the input it reads each input row once and runs on
// the matrix cores (v_mfma_f32_32x32x2f32: the ones and zeros are exact, sums are float32 as in the gather form).
//
// At graph creation the pattern is cut into aligned 32 x 32 tiles.  Tiles with at least `min_entries` stored
// entries become "dense tiles": a column-tile index and 32 words of 32 bits (word r = which columns row r has).
// Everything else stays in a residual CSR with the usual schedules.  An aggregation is then two launches:
// k_tiles writes the plain sums over the dense tiles of every row, and the gather kernels add the residual
// entries to them and finish (scaling by d_i^-1/2, activation).  Graphs without such blocks (selected tiles
// hold under a quarter of the entries) keep the single-launch gather form.
#include "common.hpp"
#include "dtypes.hpp"

namespace gcn {

namespace {

constexpr int kThreads = 256;
constexpr int kChunk = 8192;   // column tiles counted per pass: 32 KB of LDS counters

inline unsigned blocks_for(int64_t items, int per_block) { return (unsigned)((items + per_block - 1) / per_block); }

// One workgroup per row tile (32 rows).  Counts the entries of every column tile in LDS, a chunk of column
// tiles at a time, and selects the tiles with at least min_entries, in ascending column order.
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
    const int64_t r0 = rt * 32;
    const int64_t r1 = r0 + 32 < n ? r0 + 32 : n;
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

// One thread per (dense tile, row of the tile): the 32-bit word of columns that the row holds inside the tile.
__global__ void k_tile_bits(int64_t n, int64_t n_tiles, const int64_t *__restrict__ rowptr,
                            const int32_t *__restrict__ col, const int32_t *__restrict__ tile_col,
                            const int32_t *__restrict__ tile_rt, uint32_t *__restrict__ bits) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_tiles * 32) return;
    const int64_t ti = i >> 5;
    const int64_t r = (int64_t)tile_rt[ti] * 32 + (i & 31);
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

// One wave per row: the entries outside the dense tiles of the row's tile, in their order.
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
    const int64_t lo = tile_ptr[r >> 5], hi = tile_ptr[(r >> 5) + 1];
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
typedef float floatx16 __attribute__((ext_vector_type(16)));

// CB consecutive elements at p -> floats (one 4-, 8- or 16-byte load)
__device__ inline void load_elems(const float *p, float (&v)[1]) { v[0] = *p; }
__device__ inline void load_elems(const float *p, float (&v)[2]) {
    const float2 q = *reinterpret_cast<const float2 *>(p);
    v[0] = q.x;
    v[1] = q.y;
}
__device__ inline void load_elems(const float *p, float (&v)[4]) {
    const float4 q = *reinterpret_cast<const float4 *>(p);
    v[0] = q.x;
    v[1] = q.y;
    v[2] = q.z;
    v[3] = q.w;
}
// the same for bfloat16 rows (a 2-, 4- or 8-byte load), widened exactly
__device__ inline void load_elems(const bf16_t *p, float (&v)[1]) { v[0] = widen(*p); }
__device__ inline void load_elems(const bf16_t *p, float (&v)[2]) {
    typedef bf16_t bvec2 __attribute__((ext_vector_type(2)));
    const bvec2 q = *reinterpret_cast<const bvec2 *>(p);
    v[0] = (float)q[0];
    v[1] = (float)q[1];
}
__device__ inline void load_elems(const bf16_t *p, float (&v)[4]) {
    typedef bf16_t bvec4 __attribute__((ext_vector_type(4)));
    const bvec4 q = *reinterpret_cast<const bvec4 *>(p);
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = (float)q[i];
}
__device__ inline void store_elems_raw(float *p, const float (&v)[1]) { *p = v[0]; }
__device__ inline void store_elems_raw(float *p, const float (&v)[2]) {
    *reinterpret_cast<float2 *>(p) = make_float2(v[0], v[1]);
}
__device__ inline void store_elems_raw(float *p, const float (&v)[4]) {
    *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
}

// One workgroup (4 waves) per row tile: out[32 rt .. 32 rt + 32, 0 .. cols) = sum over the row tile's dense
// tiles of  bits (32 x 32, zero/one)  x  t[32 ct .. 32 ct + 32, 0 .. cols).
// A wave covers 32 * CB columns: lane l reads the CB consecutive elements CB (l % 32) .. of a row of t with one
// load (a half wave reads 128 * CB contiguous bytes) and keeps CB accumulator blocks, block j holding the output
// columns congruent j modulo CB of its span.  One MFMA step takes two columns k = 2 kk + l / 32 of the tile: lane
// l supplies bit k of row l % 32's word and, for block j, its j-th loaded element of row 32 ct + k.
// WB (1 or 2) waves stand side by side over the columns; the KS = 4 / WB waves that share a span take every KS-th
// tile of the row tile and their partial sums meet in LDS in fixed order.
// Rows of t past the matrix (only in the last column tile) read the all-zero row n; their bits are zero.
// Lanes whose columns lie past cols read column 0 instead and their results are never stored.
// The loads of a tile are unconditional and go to one of two register sets in turn, so the loads of the next
// tile are in flight while the matrix cores work on the current one.
// NARROW: every byte of t is addressable with a 32-bit offset.
template <typename TIn, int CB, int WB, bool NARROW, int OCC>
__global__ __launch_bounds__(kThreads, OCC) void k_tiles(const int64_t *__restrict__ tile_ptr,
                                                    const int32_t *__restrict__ tile_col,
                                                    const uint32_t *__restrict__ bits, int64_t n, int n_rt,
                                                    const TIn *__restrict__ t, int ld_t, float *__restrict__ out,
                                                    int ld_out, int cols) {
    constexpr int KS = 4 / WB;
    static_assert(WB == 1 || WB == 2, "one or two waves side by side");
    __shared__ float part[(KS - 1) * WB][CB * 16][64];
    const int lane = threadIdx.x & 63, half = lane >> 5, ln = lane & 31;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wb = wave % WB, ks = wave / WB;
    const int per_xcd = (n_rt + kXcds - 1) / kXcds;
    const int rt = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;   // each XCD one contiguous run of row tiles
    if (blockIdx.x / kXcds >= per_xcd || rt >= n_rt) return;
    const int c0 = (wb * 32 + ln) * CB;       // first of this lane's CB columns
    const bool cok = c0 < cols;               // cols is a multiple of 8, so all CB columns or none
    const uint32_t cbytes = (cok ? (uint32_t)c0 : 0u) * (uint32_t)sizeof(TIn);
    floatx16 acc[CB];
#pragma unroll
    for (int j = 0; j < CB; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;

    const uint32_t row_bytes = (uint32_t)ld_t * (uint32_t)sizeof(TIn);
    const int last_row = (int)n;
    // ti: a tile of this row tile (always a valid one).  Nothing here waits for a loaded value.
    auto load_tile = [&](int64_t ti, float (&b)[16][CB], uint32_t &w) {
        const int row0 = tile_col[ti] * 32 + half;
        w = bits[ti * 32 + ln];
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            int row = row0 + 2 * kk;
            row = row < last_row ? row : last_row;
            const char *p = reinterpret_cast<const char *>(t);
            if (NARROW) p += (uint32_t)row * row_bytes + cbytes;
            else p += (uint64_t)(uint32_t)row * row_bytes + cbytes;
            load_elems(reinterpret_cast<const TIn *>(p), b[kk]);
        }
    };
    auto multiply = [&](const float (&b)[16][CB], uint32_t w) {
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            const float a = ((w >> (2 * kk + half)) & 1u) ? 1.0f : 0.0f;
#pragma unroll
            for (int j = 0; j < CB; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b[kk][j], acc[j], 0, 0, 0);
        }
    };

    const int64_t tb = tile_ptr[rt], te = tile_ptr[rt + 1];
    const int64_t first = tb + ks;
    const int64_t count = first < te ? (te - first + KS - 1) / KS : 0;   // tiles of this wave
    if (count > 0) {
        const int64_t last = first + (count - 1) * KS;
        float b0[16][CB], b1[16][CB];
        uint32_t w0, w1;
        load_tile(first, b0, w0);
        int64_t i = 0;
        for (; i + 1 < count; i += 2) {   // tiles i and i + 1 both exist
            const int64_t t1 = first + (i + 1) * KS, t2 = first + (i + 2) * KS;
            // The scheduling barriers keep this order: without them the compiler sinks the loads below the matrix
            // instructions and then waits for them at once.  The body has no branch for the same reason (with
            // one, the compiler folds the two register sets into one and the overlap is gone).
            load_tile(t1, b1, w1);
            __builtin_amdgcn_sched_barrier(0);
            multiply(b0, w0);
            __builtin_amdgcn_sched_barrier(0);
            load_tile(t2 <= last ? t2 : last, b0, w0);   // past the end: the last tile again, never multiplied
            __builtin_amdgcn_sched_barrier(0);
            multiply(b1, w1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (i < count) multiply(b0, w0);   // odd count: the last tile waits in the first set
    }
    if (ks > 0) {
#pragma unroll
        for (int j = 0; j < CB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) part[(ks - 1) * WB + wb][j * 16 + v][lane] = acc[j][v];
    }
    __syncthreads();
    if (ks > 0) return;
#pragma unroll
    for (int s = 1; s < KS; ++s)
#pragma unroll
        for (int j = 0; j < CB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][v] += part[(s - 1) * WB + wb][j * 16 + v][lane];
    // accumulator element v of lane l: row 8 (v / 4) + 4 (l / 32) + v % 4; block j: column c0 + j
    if (!cok) return;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int64_t row = (int64_t)rt * 32 + 8 * (v / 4) + 4 * half + (v % 4);
        float o[CB];
#pragma unroll
        for (int j = 0; j < CB; ++j) o[j] = acc[j][v];
        if (row < n) store_elems_raw(out + row * ld_out + c0, o);
    }
}

}  // namespace

size_t tiles_capacity(int64_t entries) { return (size_t)(entries / kTileMinEntriesFloor) + 1; }

int tiles_select(int64_t n, const int64_t *rowptr, const int32_t *col, int min_entries, TileBuffers &tb,
                 int64_t *blocksum, hipStream_t st) {
    if (min_entries < kTileMinEntriesFloor || min_entries > 1024) {
        set_error("dense tiles: the entry threshold must lie in [%d, 1024]", kTileMinEntriesFloor);
        return GCN_EINVAL;
    }
    const int64_t n_ct = tb.n_rt;
    int rc = fill_zero(tb.totals, sizeof(unsigned long long), st);
    if (rc) return rc;
    k_tile_select<false><<<dim3((unsigned)tb.n_rt), dim3(kThreads), 0, st>>>(n, n_ct, rowptr, col, min_entries,
                                                                              tb.tile_cnt, nullptr, nullptr, nullptr,
                                                                              tb.totals);
    GCN_LAUNCH_CHECK();
    rc = exclusive_scan_i32(tb.n_rt, tb.tile_cnt, tb.tile_ptr, blocksum, st);
    if (rc) return rc;
    k_tile_select<true><<<dim3((unsigned)tb.n_rt), dim3(kThreads), 0, st>>>(n, n_ct, rowptr, col, min_entries,
                                                                             nullptr, tb.tile_ptr, tb.tile_col,
                                                                             tb.tile_rt, nullptr);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int tiles_build(int64_t n, const int64_t *rowptr, const int32_t *col, int64_t n_tiles, TileBuffers &tb,
                PrepBuffers &res, hipStream_t st) {
    if (n_tiles > 0) {
        k_tile_bits<<<dim3(blocks_for(n_tiles * 32, kThreads)), dim3(kThreads), 0, st>>>(n, n_tiles, rowptr, col,
                                                                                         tb.tile_col, tb.tile_rt,
                                                                                         tb.bits);
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

int tiles_launch(const SpmmArgs &a, float *dst, int ld_dst, bool beside_gather, hipStream_t st) {
    if (a.cols > 256) {
        set_error("dense tiles: at most 256 columns");
        return GCN_EINVAL;
    }
    const int n_rt = (int)a.n_rt;
    const unsigned grid = (unsigned)((n_rt + kXcds - 1) / kXcds * kXcds);
    float *out = dst;
    const size_t es = a.t_dtype == GCN_BF16 ? 2 : 4;
    const bool narrow = (uint64_t)(a.n + 1) * (uint64_t)a.ld_t * es <= 0xffffffffull;
#define GCN_TILES_T(TIn, CB, WB, OCC)                                                                                 \
    do {                                                                                                              \
        const TIn *t = static_cast<const TIn *>(a.t);                                                                 \
        if (narrow)                                                                                                   \
            k_tiles<TIn, CB, WB, true, OCC><<<dim3(grid), dim3(kThreads), 0, st>>>(                                   \
                a.tile_ptr, a.tile_col, a.bits, a.n, n_rt, t, a.ld_t, out, ld_dst, a.cols);                         \
        else                                                                                                          \
            k_tiles<TIn, CB, WB, false, OCC><<<dim3(grid), dim3(kThreads), 0, st>>>(                                  \
                a.tile_ptr, a.tile_col, a.bits, a.n, n_rt, t, a.ld_t, out, ld_dst, a.cols);                         \
    } while (0)
#define GCN_TILES(CB, WB, OCC)                                                                                        \
    do {                                                                                                              \
        if (a.t_dtype == GCN_BF16) GCN_TILES_T(bf16_t, CB, WB, OCC);                                                  \
        else GCN_TILES_T(float, CB, WB, OCC);                                                                         \
    } while (0)
    // Measured on a 47.5 k-vertex partition with 43 k dense tiles: four column blocks per wave at two waves per
    // SIMD beat one wave per SIMD (a second workgroup covers the first one's start and end) and two blocks per wave.
    if (a.cols <= 32) GCN_TILES(1, 1, 4);
    else if (a.cols <= 64) GCN_TILES(2, 1, 3);
    else if (a.cols <= 128) {
        // beside the gather kernel the smaller form (174 registers, 16 KB of LDS) finds room on a CU sooner
        if (beside_gather) GCN_TILES(2, 2, 3);
        else GCN_TILES(4, 1, 2);
    }
    else GCN_TILES(4, 2, 2);
#undef GCN_TILES
#undef GCN_TILES_T
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

}  // namespace gcn

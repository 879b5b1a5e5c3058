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
#include <algorithm>
#include <vector>

#include "common.hpp"
#include "dtypes.hpp"

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

// two bfloat16 (the upper halves of two float32 encodings) in one word: a in the low half, b in the high half
__device__ inline uint32_t pack_upper(uint32_t a, uint32_t b) {
    return __builtin_amdgcn_perm(b, a, 0x07060302u);   // bytes 2, 3 of a below bytes 2, 3 of b: one instruction
}

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

// Bits sh .. sh + 7 of w -> eight bfloat16 ones and zeros (bit sh + i -> element i).
__device__ inline bf16x8 expand_bits(uint32_t w, int sh) {
    const uint32_t byte = (w >> sh) & 0xffu;
    const uint32_t z = byte | (byte << 15);   // even bits stay in the low half, odd bits land in the high half
    union {
        uint32_t u[4];
        bf16x8 v;
    } r;
    // bit 2q of z -> 0x3F80 (bfloat16 one) in the low half, bit 2q + 16 -> the same in the high half
    r.u[0] = __umul24(z & 0x00010001u, 0x3F80u);
    r.u[1] = __umul24(z & 0x00040004u, 0x0FE0u);
    r.u[2] = __umul24(z & 0x00100010u, 0x03F8u);
    r.u[3] = __umul24(z & 0x00400040u, 0x00FEu);
    return r.v;
}

// One workgroup (4 waves) per work item = a run of dense tiles of one row block (kTileRows output rows):
//   dst[rows of the block, col0 .. col0 + 32 NB) = sum over the run's tiles of
//        bits (kTileRows x 32, zero/one)  x  t[32 ct .. 32 ct + 32, col0 .. col0 + 32 NB).
// Per tile, the waves load the 32 x 32 NB slab of t together (a thread: 8 consecutive rows of 2 columns), split
// it into bfloat16 planes and leave them in LDS in the order the matrix instruction wants its second operand:
// for every column the 8 consecutive-k values of a k-octet in one 16-byte unit.  Then wave (wm, wn) multiplies
// the bits of its SUB row tiles (32 rows each) with the planes of its JW column blocks: per 16-deep k-step one
// first operand per row tile, expanded from the bit words in registers, and one 16-byte LDS read per plane and
// column block.  Two LDS buffers: the slab of the next tile is converted and stored while the current one is
// multiplied (the conversion's instructions sit between the matrix instructions, which run in their shadow),
// its loads were issued three tiles earlier; one barrier per tile; no branch inside a step.
// Rows of t past the matrix (only in the last column tile) read the all-zero row n; their bits are zero.
// Threads whose columns lie at or past `cols` read column 0 instead; such columns are never stored.
struct TileItem {
    int32_t rb;      // row block
    int32_t first;   // index of the run's first dense tile
    int32_t count;   // tiles in the run (0: the block has none and its sums are zero)
    int32_t slot;    // -1: the sums go to the output rows; k >= 0: to block k of the partial-sum buffer
};

template <typename TIn, int NB>
__global__ __launch_bounds__(kThreads, 3) void k_tiles(const TileItem *__restrict__ items,
                                                       const int32_t *__restrict__ tile_col,
                                                       const uint32_t *__restrict__ bits, int64_t n,
                                                       const TIn *__restrict__ t, int ld_t, float *__restrict__ out,
                                                       int ld_out, float *__restrict__ partial, int cols) {
    constexpr int P = Planes<TIn>::kCount;
    constexpr int JW = NB >= 2 ? 2 : 1;            // column blocks (of 32) per wave
    constexpr int WN = NB / JW, WM = 4 / WN;       // waves side by side over the columns / stacked over the rows
    constexpr int SUB = kTileRows / 32 / WM;       // row tiles of 32 per wave
    constexpr int ROW_UNITS = 32 * NB;             // 16-byte units per k-octet of one plane: one per column
    constexpr int UNITS = 4 * ROW_UNITS;
    constexpr bool ALL_LOAD = 16 * NB * 4 == kThreads;   // every thread has a piece of the slab
    static_assert(NB == 1 || NB == 2 || NB == 4, "32, 64 or 128 columns per workgroup");
    __shared__ uint4 planes[2][P][UNITS];
    const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, l32 = lane & 31;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave % WN, wm = wave / WN;
    // workgroup b runs on XCD b mod 8 and takes place b / 8 of that XCD's sub-list (gridDim.x = 8 x its length)
    const TileItem item = items[(blockIdx.x % kXcds) * (gridDim.x / kXcds) + blockIdx.x / kXcds];
    if (item.rb < 0) return;                       // an unused place
    const int col0 = blockIdx.y * 128;             // a second row of workgroups takes columns 128 .. 255

    // loader role: k-octet kg (rows 8 kg .. 8 kg + 7 of the slab), columns 2 c2 and 2 c2 + 1 of the span
    const int c2 = tid % (16 * NB), kg = tid / (16 * NB);
    const bool loader = ALL_LOAD || kg < 4;        // whole waves either way
    const int lcol = col0 + 2 * c2;
    const TIn *lbase = t + (lcol < cols ? lcol : 0);
    const int last_row = (int)n;
    const int64_t first = item.first;
    const int count = item.count;

    struct Stage {
        uint32_t r[8][2];
        uint32_t w[SUB];
    };
    // Loads of tile i (clamped into the run, so they are always valid): the slab piece and this wave's bit words;
    // lane l holds the word of row l % 32 of each of its row tiles.  The tile's column index was fetched by the
    // fill before (ct_next), so no load here waits for another.
    int ct_next = tile_col[first];
    auto fill = [&](int i, Stage &st) {
        const int64_t ti = first + (i < count ? i : count - 1);
        const int ct = ct_next;
        ct_next = tile_col[first + (i + 1 < count ? i + 1 : count - 1)];
        if (loader) {
            const int row0 = ct * 32 + kg * 8;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                int row = row0 + k;
                row = row < last_row ? row : last_row;
                load_pair(lbase + (int64_t)row * ld_t, st.r[k]);
            }
        }
#pragma unroll
        for (int u = 0; u < SUB; ++u) st.w[u] = bits[ti * kTileRows + (wm * SUB + u) * 32 + l32];
    };
    auto convert = [&](const Stage &st, int c, uint4 (&o)[P]) {
        uint32_t x[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) x[k] = st.r[k][c];
        split_column<P>(x, o);
    };
    auto store_units = [&](int buf, int c, const uint4 (&o)[P]) {
        if (loader) {
#pragma unroll
            for (int p = 0; p < P; ++p) planes[buf][p][kg * ROW_UNITS + 2 * c2 + c] = o[p];
        }
    };

    f32x16 acc[SUB][JW];
#pragma unroll
    for (int u = 0; u < SUB; ++u)
#pragma unroll
        for (int j = 0; j < JW; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[u][j][v] = 0.0f;

    if (count > 0) {
        // Three register stages: while tile i is multiplied, the slab of tile i + 1 is converted from registers and
        // the loads of tiles i + 2 and i + 3 are in flight (a tile's arithmetic is a fraction of a load's latency).
        Stage s0, s1, s2;
        // free_st holds tile i's bit words (its slab is in LDS already), next_st tile i + 1
        auto step = [&](int i, Stage &free_st, const Stage &next_st) {
            uint32_t w_cur[SUB];
#pragma unroll
            for (int u = 0; u < SUB; ++u) w_cur[u] = free_st.w[u];
            fill(i + 3, free_st);
            const int buf = i & 1;
            uint4 o0[P], o1[P];
            union {
                uint4 q;
                bf16x8 v;
            } b[2][JW][P];
            // all LDS reads of the step first: the matrix instructions then follow each other without a wait
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int j = 0; j < JW; ++j)
#pragma unroll
                    for (int p = 0; p < P; ++p)
                        b[s][j][p].q = planes[buf][p][(2 * s + h) * ROW_UNITS + 32 * (wn * JW + j) + l32];
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                bf16x8 a[SUB];
#pragma unroll
                for (int u = 0; u < SUB; ++u) a[u] = expand_bits(w_cur[u], 16 * s + 8 * h);
                // plane-major: consecutive matrix instructions go to different accumulators
#pragma unroll
                for (int p = 0; p < P; ++p)
#pragma unroll
                    for (int u = 0; u < SUB; ++u)
#pragma unroll
                        for (int j = 0; j < JW; ++j)
                            acc[u][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u], b[s][j][p].v, acc[u][j], 0, 0, 0);
                // the next tile's slab, one of this thread's two columns per k-step, in the shadow of the above
                if (s == 0) convert(next_st, 0, o0);
                else convert(next_st, 1, o1);
            }
            store_units(buf ^ 1, 0, o0);
            store_units(buf ^ 1, 1, o1);
            __syncthreads();   // tile i + 1 is in LDS; nobody reads the buffer of tile i any more
        };
        fill(0, s0);
        fill(1, s1);
        fill(2, s2);
        {
            uint4 o0[P], o1[P];
            convert(s0, 0, o0);
            convert(s0, 1, o1);
            store_units(0, 0, o0);
            store_units(0, 1, o1);
        }
        __syncthreads();
        for (int i = 0; i < count; i += 3) {   // count is the same for the whole workgroup: the barriers line up
            step(i, s0, s1);
            if (i + 1 < count) step(i + 1, s1, s2);
            if (i + 2 < count) step(i + 2, s2, s0);
        }
    }
    // accumulator element v of lane l: row 8 (v / 4) + 4 (l / 32) + v % 4 of the row tile, column l % 32 of the block
    float *dst = item.slot < 0 ? out : partial + (int64_t)item.slot * kTileRows * ld_out;
    const int64_t base_row = item.slot < 0 ? (int64_t)item.rb * kTileRows : 0;
    const int64_t rows_left = n - (int64_t)item.rb * kTileRows;   // rows of this block inside the matrix
#pragma unroll
    for (int j = 0; j < JW; ++j) {
        const int col = col0 + 32 * (wn * JW + j) + l32;
        if (col < cols) {
#pragma unroll
            for (int u = 0; u < SUB; ++u)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = (wm * SUB + u) * 32 + 8 * (v / 4) + 4 * h + (v % 4);
                    if (row < rows_left) dst[(base_row + row) * ld_out + col] = acc[u][j][v];
                }
        }
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
    for (int k = 0; k < f.slots; ++k) {
        const float4 q =
            *reinterpret_cast<const float4 *>(partial + ((int64_t)(f.slot0 + k) * kTileRows + row) * ld_out + c0);
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
    return (size_t)kXcds * (size_t)(2 * n_rb + tile_capacity / kTileRunMin + 16);   // eight padded sub-lists
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

// The work items of the product, from the number of dense tiles of every row block (tile_ptr on the host).  A row
// block is one item unless it holds far more tiles than the average workgroup would get with every resident
// workgroup slot busy; then its tiles are cut into runs of about that many, the first run writing the output rows
// and the others partial sums that k_tiles_fold adds in run order.
// Order: workgroup b runs on XCD b mod 8 (each XCD has its own L2), so the item list is laid out as eight
// sub-lists, items[x * per_xcd + i] for workgroup 8 i + x.  The sub-lists are contiguous pieces, holding about
// equal numbers of tiles, of the sequence: one-item blocks in row order (the blocks of one community read the
// same input rows and now meet in one L2), then the runs of the cut blocks, runs with the same position in their
// block next to each other (they read the same input rows too).  Unused places hold rb = -1.
int tiles_plan(const std::vector<int64_t> &tile_ptr, TileBuffers &tb, hipStream_t st) {
    const int64_t n_rb = (int64_t)tile_ptr.size() - 1;
    const int64_t total = tile_ptr[n_rb];
    constexpr int64_t kSlots = 768;   // three workgroups on each of 256 compute units
    int64_t run = (total + kSlots - 1) / kSlots;
    if (run < kTileRunMin) run = kTileRunMin;
    std::vector<TileItem> seq, cut;
    std::vector<int> cut_pos;   // position of a run inside its block
    std::vector<TileFold> folds;
    int32_t slots = 0;
    for (int64_t rb = 0; rb < n_rb; ++rb) {
        const int64_t first = tile_ptr[rb], cnt = tile_ptr[rb + 1] - first;
        if (cnt * 2 <= run * 3) {
            seq.push_back({(int32_t)rb, (int32_t)first, (int32_t)cnt, -1});
            continue;
        }
        const int64_t parts = (cnt + run - 1) / run;
        folds.push_back({(int32_t)rb, slots, (int32_t)(parts - 1), 0});
        for (int64_t k = 0; k < parts; ++k) {
            const int64_t b = first + cnt * k / parts, e = first + cnt * (k + 1) / parts;
            cut.push_back({(int32_t)rb, (int32_t)b, (int32_t)(e - b), k == 0 ? -1 : slots++});
            cut_pos.push_back((int)k);
        }
    }
    std::vector<size_t> order(cut.size());
    for (size_t i = 0; i < order.size(); ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](size_t x, size_t y) { return cut_pos[x] < cut_pos[y]; });
    for (size_t i : order) seq.push_back(cut[i]);
    // eight contiguous pieces of about equal numbers of tiles (an item counts as at least one)
    int64_t weight = 0;
    for (const TileItem &it : seq) weight += it.count > 0 ? it.count : 1;
    std::vector<size_t> start(kXcds + 1, seq.size());
    start[0] = 0;
    {
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
    }
    size_t per_xcd = 0;
    for (int x = 0; x < kXcds; ++x) per_xcd = std::max(per_xcd, start[x + 1] - start[x]);
    std::vector<TileItem> items(per_xcd * kXcds, TileItem{-1, 0, 0, -1});
    for (int x = 0; x < kXcds; ++x)
        for (size_t i = start[x]; i < start[x + 1]; ++i) items[x * per_xcd + (i - start[x])] = seq[i];
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

int tiles_launch(const SpmmArgs &a, float *dst, int ld_dst, hipStream_t st) {
    if (a.cols > 256 || a.n_items < 1 || (a.n_slots > 0 && !a.tile_partial)) {
        set_error("dense tiles: at most 256 columns, and a partial-sum buffer when runs were cut");
        return GCN_EINVAL;
    }
    const dim3 grid((unsigned)a.n_items, a.cols > 128 ? 2u : 1u);
    const TileItem *items = reinterpret_cast<const TileItem *>(a.tile_items);
#define GCN_TILES(NB)                                                                                                 \
    do {                                                                                                              \
        if (a.t_dtype == GCN_BF16)                                                                                    \
            k_tiles<bf16_t, NB><<<grid, dim3(kThreads), 0, st>>>(items, a.tile_col, a.bits, a.n,                     \
                                                                  static_cast<const bf16_t *>(a.t), a.ld_t, dst,     \
                                                                  ld_dst, a.tile_partial, a.cols);                    \
        else                                                                                                          \
            k_tiles<float, NB><<<grid, dim3(kThreads), 0, st>>>(items, a.tile_col, a.bits, a.n,                      \
                                                                 static_cast<const float *>(a.t), a.ld_t, dst,       \
                                                                 ld_dst, a.tile_partial, a.cols);                     \
    } while (0)
    if (a.cols <= 32) GCN_TILES(1);
    else if (a.cols <= 64) GCN_TILES(2);
    else GCN_TILES(4);
#undef GCN_TILES
    GCN_LAUNCH_CHECK();
    if (a.n_folds > 0) {
        const int64_t threads = (int64_t)a.n_folds * kTileRows * (a.cols / 4);
        k_tiles_fold<<<dim3(blocks_for(threads, kThreads)), dim3(kThreads), 0, st>>>(
            reinterpret_cast<const TileFold *>(a.tile_folds), a.n_folds, a.n, dst, ld_dst, a.tile_partial, a.cols);
        GCN_LAUNCH_CHECK();
    }
    return GCN_OK;
}

}  // namespace gcn

// Aggregation  Z = A_hat T  (the sparse product of Section 4.1's layer rule; the nnz(A) F term of the
// cost model in Section 5.4), also used unchanged for the backward pass because A_hat is symmetric.
//
// The factor d_j^-1/2 of A_hat_ij = d_i^-1/2 d_j^-1/2 is already folded into the rows of the input
// (its producer scales row j once), so a row of the output is a plain sum of gathered input rows
// times d_i^-1/2.  No value array is read: 4 bytes of column index per nonzero.  Entries past the
// end of a row are replaced by column n, an all-zero input row, so inner loops need no lane masks.
//
// A group of LPR lanes covers one input row with one 16-byte load per lane (4 float32 or 8 bfloat16
// elements; LPR * that >= leading dimension), so every load instruction moves whole rows, contiguous
// in memory.  Sums are float32 whatever the storage type.
//   heavy rows (degree >= kHeavyDegree): one wave per output row; its 64 / LPR lane groups take
//     interleaved neighbours, column indices are wave-uniform and travel through the scalar path;
//     the groups' partial sums meet in a cross-lane reduction at the end.
//   light rows: one lane group per output row (64 / LPR rows per wave); each lane fetches one column
//     index (coalesced) and the group hands them round with cross-lane reads.
// Workgroup ids are dealt round-robin over the XCDs, so block ids are remapped to give each XCD one
// contiguous range of rows: neighbouring rows share neighbours, and each XCD has its own L2.
#include "common.hpp"
#include "dtypes.hpp"
#include "epilogue.hpp"

namespace gcn {

namespace {

constexpr int kThreads = 256;

typedef Activation Epi;

__device__ inline float finish(float v, const Epi &ep, int64_t row, int c) { return activate(v, ep, row, c); }

// The lane's piece of output row r (columns sub * V ...), scaled by d = d_r^-1/2 and finished.
// The sums that the dense-tile launch left in the output (float32 outputs only; never asked for with bfloat16).
template <int V>
__device__ inline void add_stored(const float *p, float (&o)[V]) {
#pragma unroll
    for (int i = 0; i < V; i += 4) {
        const float4 q = *reinterpret_cast<const float4 *>(p + i);
        o[i] += q.x;
        o[i + 1] += q.y;
        o[i + 2] += q.z;
        o[i + 3] += q.w;
    }
}
template <int V>
__device__ inline void add_stored(const bf16_t *, float (&)[V]) {}

// mode: a SpmmFinish value
template <typename TOut, int V>
__device__ inline void store_row_piece(TOut *__restrict__ out, int ld_out, int r, int sub, const float (&a)[V],
                                       const float *__restrict__ dinv, const Epi &ep, int mode) {
    const int c0 = sub * V;
    float o[V];
#pragma unroll
    for (int i = 0; i < V; ++i) o[i] = a[i];
    if (mode == kFinishAddStored) add_stored<V>(out + (int64_t)r * ld_out + c0, o);
    if (mode != kFinishPlainSum) {
        const float d = dinv[r];
#pragma unroll
        for (int i = 0; i < V; ++i) o[i] = finish(o[i] * d, ep, r, c0 + i);
    }
    store_elems<V>(out + (int64_t)r * ld_out + c0, o);
}

// One 16-byte piece of input row c: byte offset c * row_bytes + lane_bytes from t.  With NARROW the
// whole input is below 4 GiB and the offset is formed in 32 bits (scalar base + 32-bit lane offset).
template <bool NARROW, typename TIn, int V>
__device__ inline void load_piece(const TIn *__restrict__ t, int c, uint32_t row_bytes, uint32_t lane_bytes,
                                  float (&v)[V]) {
    if (NARROW) {
        const uint32_t off = (uint32_t)c * row_bytes + lane_bytes;
        unpack16(reinterpret_cast<const TIn *>(reinterpret_cast<const char *>(t) + off), v);
    } else {
        const uint64_t off = (uint64_t)(uint32_t)c * row_bytes + lane_bytes;
        unpack16(reinterpret_cast<const TIn *>(reinterpret_cast<const char *>(t) + off), v);
    }
}

template <int V>
__device__ inline void addv(float (&a)[V], const float (&v)[V]) {
#pragma unroll
    for (int i = 0; i < V; ++i) a[i] += v[i];
}

// block id -> position in the row range, so that XCD x (block ids congruent x mod 8) walks one
// contiguous eighth of the range
__device__ inline int xcd_contiguous_block(int nblocks) {
    const int per_xcd = (nblocks + kXcds - 1) / kXcds;
    return (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
}

// Sum of the input rows col[beg .. end) into two interleaved accumulators, for one wave whose 64 / LPR lane
// groups take interleaved entries: group g takes entries e + u * GPW + g, u = 0..U-1, of every step.  beg and end
// are wave-uniform, so the column indices come through the scalar path; they are fetched one step ahead (the
// read past `end` stays inside col + its slack, its values are unused).  Entries at or past `end` in the
// last, partial step are replaced by the all-zero row.
template <typename TIn, int LPR, int U, bool NARROW, int V>
__device__ inline void gather_sum(const int32_t *__restrict__ col, int64_t beg, int64_t end, int zero_row,
                                  const TIn *__restrict__ t, uint32_t row_bytes, uint32_t lane_bytes, int grp,
                                  float (&acc0)[V], float (&acc1)[V]) {
    constexpr int GPW = 64 / LPR;
    constexpr int STEP = GPW * U;
    static_assert(STEP <= kColSlack, "the index prefetch may run one step past the end of col");
    auto fetch_indices = [&](int (&c)[U], int64_t e) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (GPW == 1) {
                c[u] = col[e + u];
            } else if (GPW == 2) {
                const int c0 = col[e + 2 * u], c1 = col[e + 2 * u + 1];
                c[u] = grp ? c1 : c0;
            } else {
                c[u] = col[e + u * GPW + grp];
            }
        }
    };
    const int64_t full_end = beg + (end - beg) / STEP * STEP;
    int c[U];
    fetch_indices(c, beg);
    for (int64_t e = beg; e < full_end; e += STEP) {
        int cn[U];
        fetch_indices(cn, e + STEP);
        float v[U][V];
#pragma unroll
        for (int u = 0; u < U; ++u) load_piece<NARROW>(t, c[u], row_bytes, lane_bytes, v[u]);
#pragma unroll
        for (int u = 0; u < U; u += 2) {
            addv(acc0, v[u]);
            addv(acc1, v[u + 1]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) c[u] = cn[u];
    }
    if (full_end < end) {
        float v[U][V];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t pos = full_end + u * GPW + grp;
            const int cc = pos < end ? c[u] : zero_row;
            load_piece<NARROW>(t, cc, row_bytes, lane_bytes, v[u]);
        }
#pragma unroll
        for (int u = 0; u < U; u += 2) {
            addv(acc0, v[u]);
            addv(acc1, v[u + 1]);
        }
    }
}

// ------------------------------------------------------------------------------------------------ heavy rows
template <typename TIn, typename TOut, int LPR, int U, bool NARROW>
__global__ __launch_bounds__(kThreads) void k_spmm_wave(const int64_t *__restrict__ rowptr,
                                                        const int32_t *__restrict__ col,
                                                        const int32_t *__restrict__ perm,
                                                        const int32_t *__restrict__ xcd_start,
                                                        const float *__restrict__ dinv, int zero_row,
                                                        const TIn *__restrict__ t, int ld_t,
                                                        TOut *__restrict__ out, int ld_out, int cols, Epi ep, int mode) {
    constexpr int V = Piece<TIn>::kElems;
    constexpr int GPW = 64 / LPR;      // lane groups per wave = neighbours per load instruction
    constexpr int STEP = GPW * U;      // neighbours per unrolled step
    static_assert(STEP <= kColSlack, "the index prefetch may run one step past the end of col");
    constexpr int RPB = kThreads / 64;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int grp = lane / LPR, sub = lane % LPR;
    // XCD x (block ids congruent x mod 8) walks its own contiguous run of the schedule; the runs hold about the
    // same number of entries each, so their lengths in rows differ
    const int x = blockIdx.x % kXcds;
    const int64_t s = xcd_start[x] + (int64_t)(blockIdx.x / kXcds) * RPB + wave;
    if (s >= xcd_start[x + 1]) return;
    const int r = perm[s];
    const int64_t beg = rowptr[r], end = rowptr[r + 1];
    // lanes beyond the row's width re-read its first piece (in bounds, same cache line) and store nothing
    const uint32_t lane_bytes = (sub * V < cols) ? sub * 16u : 0u;
    const uint32_t row_bytes = (uint32_t)ld_t * (uint32_t)sizeof(TIn);

    float acc0[V], acc1[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc0[i] = acc1[i] = 0.0f;
    gather_sum<TIn, LPR, U, NARROW>(col, beg, end, zero_row, t, row_bytes, lane_bytes, grp, acc0, acc1);
    float a[V];
#pragma unroll
    for (int i = 0; i < V; ++i) {
        a[i] = acc0[i] + acc1[i];
#pragma unroll
        for (int d = LPR; d < 64; d <<= 1) a[i] += __shfl_xor(a[i], d, 64);
    }
    if (grp == 0 && sub * V < cols) store_row_piece<TOut, V>(out, ld_out, r, sub, a, dinv, ep, mode);
}

// ------------------------------------------------------------------------------------------------ phased schedule
// For inputs a few times larger than one L2 (one partition of a distributed graph is that size): the vertex ids
// are cut into kXcds equal row ranges and kColBlocks equal column ranges.  XCD x owns the rows of row range x; each
// of its waves owns R rows for the whole kernel and keeps their sums in registers.  The work goes in kColBlocks / G
// phases of G adjacent column ranges: in a phase every wave of XCD x adds, for each of its rows, the entries whose
// columns lie in the phase's ranges (rows are sorted, so that is one contiguous segment, found through segoff).
// The XCDs start on different ranges, each right behind the ranges of its own rows and ending on them: those hold
// the rows' neighbourhood, the long pass, and right after the common start, on the short ones, all waves still
// move in step.  Waves carry similar loads (rows are dealt to waves by degree, in serpentine order), so for a
// while an XCD's gathers fall into one phase's ranges, which its L2 holds: most entries outside a row's own
// neighbourhood stop missing.  There is no synchronisation of any kind: a row never leaves its wave, and waves
// that drift apart only lose hits.  (Measured on the benchmark partition: L2 misses -54 %, time -8 %; pacing the
// waves with counters between phases removed 86 % of the misses but cost more time in waiting than it saved.)
template <typename TIn, typename TOut, int LPR, int U, int R, int G>
__global__ __launch_bounds__(kThreads) void k_spmm_phased(const int64_t *__restrict__ rowptr,
                                                          const int32_t *__restrict__ col,
                                                          const int32_t *__restrict__ segoff,
                                                          const int32_t *__restrict__ prow, int W,
                                                          const float *__restrict__ dinv, int zero_row, int64_t n,
                                                          int64_t block, const TIn *__restrict__ t, int ld_t,
                                                          TOut *__restrict__ out, int ld_out, int cols, Epi ep,
                                                          int mode) {
    constexpr int V = Piece<TIn>::kElems;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int grp = lane / LPR, sub = lane % LPR;
    const int x = blockIdx.x % kXcds;
    const int64_t q = (int64_t)(blockIdx.x / kXcds) * (kThreads / 64) + wave;   // wave number inside its XCD
    if (q >= W) return;
    const int32_t *mine = prow + ((int64_t)x * W + q) * R;   // this wave's rows (degree-balanced), -1 = none
    int rows[R];
#pragma unroll
    for (int j = 0; j < R; ++j) rows[j] = mine[j];
    const uint32_t lane_bytes = (sub * V < cols) ? sub * 16u : 0u;
    const uint32_t row_bytes = (uint32_t)ld_t * (uint32_t)sizeof(TIn);
    float acc[R][V];
#pragma unroll
    for (int j = 0; j < R; ++j)
#pragma unroll
        for (int i = 0; i < V; ++i) acc[j][i] = 0.0f;
    constexpr int kPhases = kColBlocks / G;
    const int own = kRangesPerXcd * x / G;   // the phase that holds the column ranges of this XCD's rows: the last one
    for (int s = 1; s <= kPhases; ++s) {
        const int b = (own + s) % kPhases * G;
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const int64_t r = rows[j];
            if (r >= 0) {
                const int64_t row_beg = rowptr[r];
                const int32_t *so = segoff + r * (kColBlocks + 1);
                float a1[V];
#pragma unroll
                for (int i = 0; i < V; ++i) a1[i] = 0.0f;
                gather_sum<TIn, LPR, U, true>(col, row_beg + so[b], row_beg + so[b + G], zero_row, t, row_bytes, lane_bytes,
                                              grp, acc[j], a1);
                addv(acc[j], a1);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const int64_t r = rows[j];
        if (r >= 0) {
            float a[V];
#pragma unroll
            for (int i = 0; i < V; ++i) {
                a[i] = acc[j][i];
#pragma unroll
                for (int d = LPR; d < 64; d <<= 1) a[i] += __shfl_xor(a[i], d, 64);
            }
            if (grp == 0 && sub * V < cols) store_row_piece<TOut, V>(out, ld_out, (int)r, sub, a, dinv, ep, mode);
        }
    }
}

// ------------------------------------------------------------------------------------------------ split rows
// A row with more than kSplitDegree entries would keep one wave busy long after everything else has ended (a hub of
// 150,000 entries takes 9,500 dependent steps), so such rows are cut into chunks of kChunk entries: one wave per
// chunk writes the chunk's plain sum, and k_spmm_chunk_rows adds a row's chunks in ascending order and finishes the row.
template <typename TIn, int LPR, int U, bool NARROW>
__global__ __launch_bounds__(kThreads) void k_spmm_chunks(const int64_t *__restrict__ rowptr,
                                                          const int32_t *__restrict__ col,
                                                          const int32_t *__restrict__ split_rows,
                                                          const int64_t *__restrict__ chunk_off,
                                                          const int32_t *__restrict__ chunk_srow, int64_t n_chunks,
                                                          int zero_row, const TIn *__restrict__ t, int ld_t, int cols,
                                                          float *__restrict__ chunk_sums) {
    constexpr int V = Piece<TIn>::kElems;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int grp = lane / LPR, sub = lane % LPR;
    const int64_t c = (int64_t)blockIdx.x * (kThreads / 64) + wave;
    if (c >= n_chunks) return;
    const int j = chunk_srow[c];
    const int r = split_rows[j];
    const int64_t beg = rowptr[r] + (c - chunk_off[j]) * kChunk;
    const int64_t row_end = rowptr[r + 1];
    const int64_t end = beg + kChunk < row_end ? beg + kChunk : row_end;
    const uint32_t lane_bytes = (sub * V < cols) ? sub * 16u : 0u;
    const uint32_t row_bytes = (uint32_t)ld_t * (uint32_t)sizeof(TIn);
    float acc0[V], acc1[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc0[i] = acc1[i] = 0.0f;
    gather_sum<TIn, LPR, U, NARROW>(col, beg, end, zero_row, t, row_bytes, lane_bytes, grp, acc0, acc1);
    float a[V];
#pragma unroll
    for (int i = 0; i < V; ++i) {
        a[i] = acc0[i] + acc1[i];
#pragma unroll
        for (int d = LPR; d < 64; d <<= 1) a[i] += __shfl_xor(a[i], d, 64);
    }
    if (grp == 0 && sub * V < cols) store_elems<V>(chunk_sums + c * cols + sub * V, a);
}

// One thread per (split row, four columns): the row's chunk sums in ascending order, then the row is finished
// as the other kernels finish theirs (mode: a SpmmFinish value).
template <typename TOut>
__global__ __launch_bounds__(kThreads) void k_spmm_chunk_rows(const int32_t *__restrict__ split_rows,
                                                              const int64_t *__restrict__ chunk_off, int64_t n_split,
                                                              const float *__restrict__ chunk_sums, int cols,
                                                              const float *__restrict__ dinv, TOut *__restrict__ out,
                                                              int ld_out, Epi ep, int mode) {
    const int quads = cols / 4;
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n_split * quads) return;
    const int64_t j = i / quads;
    const int c0 = (int)(i % quads) * 4;
    const int r = split_rows[j];
    float o[4] = {0.f, 0.f, 0.f, 0.f};
    for (int64_t c = chunk_off[j]; c < chunk_off[j + 1]; ++c) {
        const float4 q = *reinterpret_cast<const float4 *>(chunk_sums + c * cols + c0);
        o[0] += q.x;
        o[1] += q.y;
        o[2] += q.z;
        o[3] += q.w;
    }
    if (mode == kFinishAddStored) add_stored<4>(out + (int64_t)r * ld_out + c0, o);
    if (mode != kFinishPlainSum) {
        const float d = dinv[r];
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = finish(o[k] * d, ep, r, c0 + k);
    }
    store_elems<4>(out + (int64_t)r * ld_out + c0, o);
}

// ------------------------------------------------------------------------------------------------ light rows
template <typename TIn, typename TOut, int LPR, int U, bool NARROW>
__global__ __launch_bounds__(kThreads) void k_spmm_group(const int64_t *__restrict__ rowptr,
                                                         const int32_t *__restrict__ col,
                                                         const int32_t *__restrict__ perm,
                                                         const float *__restrict__ dinv, int zero_row,
                                                         int64_t n_rows, const TIn *__restrict__ t, int ld_t,
                                                         TOut *__restrict__ out, int ld_out, int cols, int nblocks,
                                                         Epi ep, int mode) {
    static_assert(LPR % U == 0, "one index fetch feeds a whole number of unrolled steps");
    constexpr int V = Piece<TIn>::kElems;
    constexpr int GPW = 64 / LPR;                 // rows per wave
    constexpr int RPB = (kThreads / 64) * GPW;    // rows per workgroup
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane / LPR, sub = lane % LPR;
    const int blk = xcd_contiguous_block(nblocks);
    if (blk >= nblocks) return;
    const int64_t s = (int64_t)blk * RPB + wave * GPW + grp;
    const bool live = s < n_rows;
    const uint32_t lane_bytes = (sub * V < cols) ? sub * 16u : 0u;
    const uint32_t row_bytes = (uint32_t)ld_t * (uint32_t)sizeof(TIn);
    int64_t beg = 0, end = 0;
    int r = 0;
    if (live) {
        r = perm[s];
        beg = rowptr[r];
        end = rowptr[r + 1];
    }
    float acc0[V], acc1[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc0[i] = acc1[i] = 0.0f;
    int nxt = (beg + sub < end) ? col[beg + sub] : zero_row;
    for (int64_t e = beg; e < end; e += LPR) {
        const int mine = nxt;         // entry e + sub, or the zero row past the end
        const int cnt = (end - e) < LPR ? (int)(end - e) : LPR;
        const int64_t e2 = e + LPR + sub;
        nxt = (e2 < end) ? col[e2] : zero_row;
        for (int k = 0; k < cnt; k += U) {
            int c[U];
            float v[U][V];
#pragma unroll
            for (int u = 0; u < U; ++u) c[u] = __shfl(mine, grp * LPR + k + u, 64);
#pragma unroll
            for (int u = 0; u < U; ++u) load_piece<NARROW>(t, c[u], row_bytes, lane_bytes, v[u]);
#pragma unroll
            for (int u = 0; u + 1 < U; u += 2) {
                addv(acc0, v[u]);
                addv(acc1, v[u + 1]);
            }
        }
    }
    if (live && sub * V < cols) {
        float a[V];
#pragma unroll
        for (int i = 0; i < V; ++i) a[i] = acc0[i] + acc1[i];
        store_row_piece<TOut, V>(out, ld_out, r, sub, a, dinv, ep, mode);
    }
}

// ------------------------------------------------------------------------------------------------ joining the parts
// out[r, c .. c + 4) = finish(d_r^-1/2 (sums[r, c ..] + tile_sums[r, c ..])): the gather kernel's plain sums over
// the residual entries (float32: left in out itself, sums == out) plus the tile product's sums, one thread per four
// columns.
template <typename TOut>
__global__ __launch_bounds__(kThreads) void k_join_parts(TOut *out, int ld_out, const float *sums, int ld_sums,
                                                         const float *__restrict__ tile_sums, int ld_tile,
                                                         const float *__restrict__ dinv, int64_t n, int cols, Epi ep) {
    const int quads = cols / 4;
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n * quads) return;
    const int64_t r = i / quads;
    const int c0 = (int)(i % quads) * 4;
    const float4 a = *reinterpret_cast<const float4 *>(sums + r * ld_sums + c0);
    const float4 b = *reinterpret_cast<const float4 *>(tile_sums + r * ld_tile + c0);
    const float d = dinv[r];
    float v[4];
    v[0] = finish((a.x + b.x) * d, ep, r, c0);
    v[1] = finish((a.y + b.y) * d, ep, r, c0 + 1);
    v[2] = finish((a.z + b.z) * d, ep, r, c0 + 2);
    v[3] = finish((a.w + b.w) * d, ep, r, c0 + 3);
    store_elems<4>(out + r * ld_out + c0, v);
}

// true when every byte of the input (n + 1 rows) is addressable with a 32-bit offset
inline bool narrow_ok(const SpmmArgs &a, size_t elem) {
    return (uint64_t)(a.n + 1) * (uint64_t)a.ld_t * elem <= 0xffffffffull;
}

template <typename TIn, typename TOut, int LPR, int UW, int UG>
int launch(const SpmmArgs &a, hipStream_t st) {
    Epi ep{a.epilogue == kEpiRelu ? kActRelu : kActNone, a.width, a.drop_threshold, a.keep_scale, a.drop_key};
    const bool narrow = narrow_ok(a, sizeof(TIn));
    const int zero_row = (int)a.n;
    const TIn *t = static_cast<const TIn *>(a.t);
    TOut *out = static_cast<TOut *>(a.out);
    if (a.n_heavy > 0) {
        constexpr int RPB = kThreads / 64;
        const unsigned grid = (unsigned)(kXcds * ((a.xcd_rows_max + RPB - 1) / RPB));
        if (narrow)
            k_spmm_wave<TIn, TOut, LPR, UW, true><<<dim3(grid), dim3(kThreads), 0, st>>>(
                a.rowptr, a.col, a.perm, a.xcd_start, a.dinv, zero_row, t, a.ld_t, out, a.ld_out, a.cols, ep, a.finish_mode);
        else
            k_spmm_wave<TIn, TOut, LPR, UW, false><<<dim3(grid), dim3(kThreads), 0, st>>>(
                a.rowptr, a.col, a.perm, a.xcd_start, a.dinv, zero_row, t, a.ld_t, out, a.ld_out, a.cols, ep, a.finish_mode);
        GCN_LAUNCH_CHECK();
    }
    if (a.n_split > 0) {
        const int32_t *split_rows = a.perm + a.n_heavy + a.n_light;
        const unsigned cgrid = (unsigned)((a.n_chunks + kThreads / 64 - 1) / (kThreads / 64));
        if (narrow)
            k_spmm_chunks<TIn, LPR, UW, true><<<dim3(cgrid), dim3(kThreads), 0, st>>>(
                a.rowptr, a.col, split_rows, a.chunk_off, a.chunk_srow, a.n_chunks, zero_row, t, a.ld_t, a.cols, a.chunk_sums);
        else
            k_spmm_chunks<TIn, LPR, UW, false><<<dim3(cgrid), dim3(kThreads), 0, st>>>(
                a.rowptr, a.col, split_rows, a.chunk_off, a.chunk_srow, a.n_chunks, zero_row, t, a.ld_t, a.cols, a.chunk_sums);
        GCN_LAUNCH_CHECK();
        const int64_t items = a.n_split * (a.cols / 4);
        k_spmm_chunk_rows<TOut><<<dim3((unsigned)((items + kThreads - 1) / kThreads)), dim3(kThreads), 0, st>>>(
            split_rows, a.chunk_off, a.n_split, a.chunk_sums, a.cols, a.dinv, out, a.ld_out, ep, a.finish_mode);
        GCN_LAUNCH_CHECK();
    }
    const int64_t n_light = a.n_light;
    if (n_light > 0) {
        constexpr int RPB = (kThreads / 64) * (64 / LPR);
        const int nblocks = (int)((n_light + RPB - 1) / RPB);
        const int grid = (nblocks + kXcds - 1) / kXcds * kXcds;
        if (narrow)
            k_spmm_group<TIn, TOut, LPR, UG, true><<<dim3(grid), dim3(kThreads), 0, st>>>(
                a.rowptr, a.col, a.perm + a.n_heavy, a.dinv, zero_row, n_light, t, a.ld_t, out, a.ld_out, a.cols, nblocks,
                ep, a.finish_mode);
        else
            k_spmm_group<TIn, TOut, LPR, UG, false><<<dim3(grid), dim3(kThreads), 0, st>>>(
                a.rowptr, a.col, a.perm + a.n_heavy, a.dinv, zero_row, n_light, t, a.ld_t, out, a.ld_out, a.cols, nblocks,
                ep, a.finish_mode);
        GCN_LAUNCH_CHECK();
    }
    return GCN_OK;
}

// The phased schedule applies when nearly every row is heavy, the input is larger than one L2 but one column range of it
// fits, and a wave gets at most 8 rows with the whole grid resident.  Knob "spmm_phased": -1 automatic
// (default), 0 never, 1 whenever the shape allows.
constexpr int64_t kL2Bytes = 4 << 20;
// Input rows per phase, in bytes.  Measured on the benchmark partition (time of the aggregation inside an epoch):
//   512-byte rows (float32, width 128):  1.5 MB +19 %, 3.0 MB best, 6.1 MB +14 %
//   256-byte rows (bfloat16, width 128): 1.5 MB +14 %, 3.0 MB +4 %, 6.1 MB best
//   192-byte rows (float32, width 48):   2.3 MB +6 %, 4.6 MB best, 9.1 MB +5 %
// so rows of at least 512 bytes (a lane group of 32 or 64 lanes) get up to 5 MB, narrower ones up to 6.5 MB.
// That partition keeps the vertices of a community together, so a phase's gathers fall on few of its rows.  Where
// the entries are spread evenly over the columns (the same partition with its vertex ids scrambled) a phase's rows
// must fit an L2 beside everything else: one column range of 1.5 MB per phase gave 554 epochs/s against 479 with two
// and 415 with four.
constexpr int64_t kPhaseBytesWide = 5 << 20;
constexpr int64_t kPhaseBytesNarrow = (13 << 20) / 2;
constexpr int64_t kPhaseBytesSpread = (13 << 20) / 8;

template <typename TIn, typename TOut, int LPR, int U>
bool try_phased(const SpmmArgs &a, hipStream_t st, int *rc) {
    const int64_t knob = tunable("spmm_phased", -1);
    const int W = a.phased_w, R = a.phased_r;
    if (knob == 0 || !a.segoff || !a.prow || W < 1 || !narrow_ok(a, sizeof(TIn))) return false;
    if (knob < 0 && (a.n_heavy + a.n_split) * 8 < a.n * 7) return false;   // a wave per light row wastes most of its lanes
    if (knob < 0 && a.n_split * 16 > a.n) return false;   // many very long rows: chunks balance better than whole rows
    const int64_t block = (a.n + kColBlocks - 1) / kColBlocks;
    const int64_t row_bytes = (int64_t)a.ld_t * (int64_t)sizeof(TIn);
    if (knob < 0 && ((a.n + 1) * row_bytes <= kL2Bytes || block * row_bytes > kL2Bytes - (512 << 10))) return false;
    const unsigned grid = (unsigned)(kXcds * ((W + kThreads / 64 - 1) / (kThreads / 64)));
    Epi ep{a.epilogue == kEpiRelu ? kActRelu : kActNone, a.width, a.drop_threshold, a.keep_scale, a.drop_key};
    const TIn *t = static_cast<const TIn *>(a.t);
    TOut *out = static_cast<TOut *>(a.out);
    const int zero_row = (int)a.n;
    // column ranges per phase (1, 2, 4 or 8): the most whose rows take at most kPhaseBytesWide / Narrow.  Knob "phased_group":
    // 0 = this rule.
    int64_t group = tunable("phased_group", 0);
    if (group <= 0)
        for (group = kColBlocks / 2;
             group > 1 && group * block * row_bytes >
                              (a.spread ? kPhaseBytesSpread : (LPR >= 32 ? kPhaseBytesWide : kPhaseBytesNarrow));)
            group /= 2;
#define GCN_PHASED(RR, GG)                                                                                           \
    k_spmm_phased<TIn, TOut, LPR, U, RR, GG><<<dim3(grid), dim3(kThreads), 0, st>>>(                                  \
        a.rowptr, a.col, a.segoff, a.prow, W, a.dinv, zero_row, a.n, block, t, a.ld_t, out, a.ld_out, \
        a.cols, ep, a.finish_mode)
#define GCN_PHASED_R(GG)                                                                                             \
    do {                                                                                                             \
        if (R == 4) GCN_PHASED(4, GG);                                                                               \
        else if (R == 6) GCN_PHASED(6, GG);                                                                          \
        else GCN_PHASED(8, GG);                                                                                      \
    } while (0)
    if (group >= 8) GCN_PHASED_R(8);
    else if (group >= 4) GCN_PHASED_R(4);
    else if (group >= 2) GCN_PHASED_R(2);
    else GCN_PHASED_R(1);
#undef GCN_PHASED_R
#undef GCN_PHASED
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("kernel launch failed: %s (%s:%d)", hipGetErrorString(e), __FILE__, __LINE__);
        *rc = GCN_EHIP;
    } else {
        *rc = GCN_OK;
    }
    return true;
}

inline int hip_status(hipError_t e, const char *what) {
    if (e == hipSuccess) return GCN_OK;
    set_error("%s failed: %s", what, hipGetErrorString(e));
    return GCN_EHIP;
}

template <typename TIn, typename TOut>
int launch_by_width(const SpmmArgs &a, hipStream_t st) {
    const int pieces = (a.cols + Piece<TIn>::kElems - 1) / Piece<TIn>::kElems;   // 16-byte pieces per row
    int rc = GCN_OK;
    if (pieces > 32 && try_phased<TIn, TOut, 64, 4>(a, st, &rc)) return rc;
    if (pieces > 16 && pieces <= 32 && try_phased<TIn, TOut, 32, 4>(a, st, &rc)) return rc;
    if (pieces > 4 && pieces <= 8 && try_phased<TIn, TOut, 8, 2>(a, st, &rc)) return rc;
    if (pieces > 8 && pieces <= 16 && try_phased<TIn, TOut, 16, 2>(a, st, &rc)) return rc;
    if (pieces <= 4) return launch<TIn, TOut, 4, 2, 4>(a, st);
    if (pieces <= 8) return launch<TIn, TOut, 8, 2, 8>(a, st);
    if (pieces <= 16) return launch<TIn, TOut, 16, 4, 8>(a, st);
    if (pieces <= 32) {
        const int64_t u = tunable("spmm_u", 8);
        if (u == 4) return launch<TIn, TOut, 32, 4, 8>(a, st);
        if (u == 16) return launch<TIn, TOut, 32, 16, 8>(a, st);
        return launch<TIn, TOut, 32, 8, 8>(a, st);
    }
    return launch<TIn, TOut, 64, 8, 8>(a, st);
}

}  // namespace

int spmm_launch(const SpmmArgs &a, hipStream_t st) {
    if (a.n <= 0) return GCN_OK;
    const int v_in = a.t_dtype == GCN_BF16 ? 8 : 4;
    if (a.ld_t % 8 != 0 || a.ld_out % 8 != 0 || a.cols % 8 != 0 || a.cols < 8 || a.cols > a.ld_t || a.cols > a.ld_out ||
        a.cols > 64 * v_in || a.n_heavy < 0 || a.n_light < 0 || a.n_split < 0 || a.n_heavy + a.n_light + a.n_split != a.n ||
        (a.n_heavy > 0 && (!a.xcd_start || a.xcd_rows_max < (a.n_heavy + kXcds - 1) / kXcds || a.xcd_rows_max > a.n_heavy)) ||
        (a.n_split > 0 && (!a.chunk_sums || !a.chunk_off || !a.chunk_srow || a.n_chunks < a.n_split)) || (a.t_dtype == GCN_F32 && a.out_dtype != GCN_F32)) {
        set_error("aggregation: unsupported shape (ld %d / %d, heavy %lld of %lld, types %d -> %d)", a.ld_t, a.ld_out,
                  (long long)a.n_heavy, (long long)a.n, a.t_dtype, a.out_dtype);
        return GCN_EINVAL;
    }
    const int t_all = timing_open(kTimeAggregate, a.width, st);
    SpmmArgs b = a;
    b.finish_mode = kFinishRow;
    int rc = GCN_OK;
    // side by side needs somewhere to leave the gather's plain float32 sums: the output itself, or gather_sums
    const bool overlap = a.tile_ptr && a.tile_sums && a.side && a.ev_fork && a.ev_join &&
                         (a.out_dtype == GCN_F32 || a.gather_sums) && tunable("spmm_overlap", 1) != 0;
    if (a.tile_ptr && !overlap && a.out_dtype != GCN_F32) {
        set_error("aggregation: dense tiles with a bfloat16 output need the side stream and both sum buffers");
        timing_close(t_all, st);
        return GCN_EINVAL;
    }
    // Side by side: the tile product and the gather over the residual entries on two streams, the caller's and the
    // graph's own (which one where: below).  Both kernels slow each other down through the bytes they pull from
    // the L2s (the benchmark partition: 254 us together against 195 + 98 us alone).
    hipStream_t gather_stream = st;
    // The pass that lays the input out for the tile product.  float32: before the two parts are forked (beside the
    // gather it takes three times as long, and the tile product's is the longer of the two paths).  bfloat16: at the
    // head of the tile product's own path, beside the gather (there the gather's path is the longer one: measured
    // 0.236 against 0.218 ms for the width-128 aggregation of the benchmark partition).
    const bool planes_first = a.tile_ptr && !(overlap && a.t_dtype == GCN_BF16);
    if (planes_first) rc = tiles_planes(a, st);
    if (rc != GCN_OK) {
        timing_close(t_all, st);
        return rc;
    }
    if (a.tile_ptr && overlap) {
        rc = hip_status(hipEventRecord(a.ev_fork, st), "hipEventRecord");
        if (rc == GCN_OK) rc = hip_status(hipStreamWaitEvent(a.side, a.ev_fork, 0), "hipStreamWaitEvent");
        // Which of the two goes first into the chip (the caller's stream; the other follows on the side stream): the
        // gather when it runs the phased schedule, whose grid must be resident at once (the benchmark partition:
        // 943 against 817 epochs/s), the tile product otherwise, because it is the longer of the two (the full
        // Reddit shape: 137.5 against 133.7 epochs/s).  Knob "spmm_tiles_first": -1 this rule, 0 / 1 fixed.
        const int64_t first_knob = tunable("spmm_tiles_first", -1);
        const bool tiles_first = first_knob < 0 ? a.phased_w <= 0 : first_knob != 0;
        if (rc == GCN_OK && tiles_first) {
            if (!planes_first) rc = tiles_planes(a, st);
            if (rc == GCN_OK) rc = tiles_launch(a, a.tile_sums, a.cols, st);
            gather_stream = a.side;
        } else if (rc == GCN_OK) {
            if (!planes_first) rc = tiles_planes(a, a.side);
            if (rc == GCN_OK) rc = tiles_launch(a, a.tile_sums, a.cols, a.side);
        }
        b.finish_mode = kFinishPlainSum;
        if (a.out_dtype != GCN_F32) {
            b.out = a.gather_sums;
            b.out_dtype = GCN_F32;
            b.ld_out = a.cols;
        }
    } else if (a.tile_ptr) {
        rc = tiles_launch(a, static_cast<float *>(a.out), a.ld_out, st);
        b.finish_mode = kFinishAddStored;
    }
    if (rc == GCN_OK) {
        const int t_gather = timing_open(kTimeGather, a.width, gather_stream);
        if (b.t_dtype == GCN_F32) rc = launch_by_width<float, float>(b, gather_stream);
        else if (b.out_dtype == GCN_F32) rc = launch_by_width<bf16_t, float>(b, gather_stream);
        else rc = launch_by_width<bf16_t, bf16_t>(b, gather_stream);
        timing_close(t_gather, gather_stream);
    }
    if (a.tile_ptr && overlap) {
        // join, also after an error above: the caller's stream must not run ahead of work already on the side stream
        int rc2 = hip_status(hipEventRecord(a.ev_join, a.side), "hipEventRecord");
        if (rc2 == GCN_OK) rc2 = hip_status(hipStreamWaitEvent(st, a.ev_join, 0), "hipStreamWaitEvent");
        if (rc == GCN_OK) rc = rc2;
        if (rc == GCN_OK) {
            const int t_join = timing_open(kTimeJoin, a.width, st);
            Epi ep{a.epilogue == kEpiRelu ? kActRelu : kActNone, a.width, a.drop_threshold, a.keep_scale, a.drop_key};
            const int64_t quads = a.n * (a.cols / 4);
            const dim3 grid((unsigned)((quads + kThreads - 1) / kThreads));
            if (a.out_dtype == GCN_F32)
                k_join_parts<float><<<grid, dim3(kThreads), 0, st>>>(static_cast<float *>(a.out), a.ld_out,
                                                                    static_cast<const float *>(a.out), a.ld_out,
                                                                    a.tile_sums, a.cols, a.dinv, a.n, a.cols, ep);
            else
                k_join_parts<bf16_t><<<grid, dim3(kThreads), 0, st>>>(static_cast<bf16_t *>(a.out), a.ld_out,
                                                                     a.gather_sums, a.cols, a.tile_sums, a.cols,
                                                                     a.dinv, a.n, a.cols, ep);
            rc = hip_status(hipGetLastError(), "k_join_parts launch");
            timing_close(t_join, st);
        }
    }
    timing_close(t_all, st);
    return rc;
}

}  // namespace gcn

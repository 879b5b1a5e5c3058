// Graph preparation on the GPU: validation, canonical pattern of A + I, integer degrees, D^-1/2,
// and the padded row schedule the aggregation kernels walk.
//
// A_hat = D^-1/2 (A + I) D^-1/2 is the "normalized adjacency matrix" named in the footnote to
// Section 4.1 (form of the cited Kipf-Welling model); A is the adjacency matrix of Section 2.1.
// Everything here is integer work except d^-1/2.
#include "common.hpp"

namespace gcn {

namespace {

constexpr int kThreads = 256;
constexpr int kSortCap = 4096;                 // rows up to this many entries (incl. the self-loop) are sorted in LDS
constexpr int kChunkCols = kSortCap * 32;      // longer rows: one bit per column, this many columns per pass
constexpr int kSentinel = 0x7fffffff;

// Exclusive prefix sum over the 256 threads of a workgroup, in thread order; *total = sum of all.
// Two barriers inside; every thread must call it.
__device__ inline int block_exclusive_scan(int v, int *total, int *wave_sums /* LDS, 4 ints */) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
    }
    __syncthreads();   // wave_sums may still be read by a previous call
    if (lane == 63) wave_sums[wave] = incl;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) {
        int s = wave_sums[w];
        if (w < wave) before += s;
        all += s;
    }
    *total = all;
    return before + incl - v;
}

// --------------------------------------------------------------------------------------------- validation
__global__ void k_validate_rowptr(int64_t n, int64_t nnz, const int64_t *__restrict__ rowptr, int32_t *flags) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i > n) return;
    bool bad = false;
    int64_t a = rowptr[i];
    if (i == 0 && a != 0) bad = true;
    if (i == n && a != nnz) bad = true;
    if (a < 0 || a > nnz) bad = true;
    if (i < n && rowptr[i + 1] < a) bad = true;
    if (bad) atomicOr(&flags[0], 1);
}

__global__ void k_validate_col(int64_t n, int64_t nnz, const int32_t *__restrict__ col, int32_t *flags) {
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= nnz) return;
    int32_t c = col[p];
    if (c < 0 || c >= n) atomicOr(&flags[0], 2);
}

// --------------------------------------------------------------------------------------------- canonical rows
// One workgroup per row i.  Writes the ascending, distinct columns of row i of A + I (the raw
// entries other than i, plus i once) to scratch[rowptr[i] + i ...] and their count to deg[i].
__global__ __launch_bounds__(kThreads) void k_canonical_rows(int64_t n, const int64_t *__restrict__ rowptr,
                                                             const int32_t *__restrict__ col,
                                                             int32_t *__restrict__ scratch, int32_t *__restrict__ deg) {
    __shared__ int s[kSortCap];
    __shared__ int wave_sums[4];
    const int tid = threadIdx.x;
    const int64_t i = blockIdx.x;
    const int64_t b = rowptr[i];
    const int64_t len = rowptr[i + 1] - b;
    int32_t *out = scratch + b + i;
    int running = 0;

    if (len + 1 <= kSortCap) {
        const int m = (int)len + 1;
        int P = 2;
        while (P < m) P <<= 1;
        for (int t = tid; t < P; t += kThreads) s[t] = t < len ? col[b + t] : (t == len ? (int)i : kSentinel);
        __syncthreads();
        // bitonic sort, ascending
        for (int k = 2; k <= P; k <<= 1) {
            for (int j = k >> 1; j > 0; j >>= 1) {
                for (int t = tid; t < P; t += kThreads) {
                    int x = t ^ j;
                    if (x > t) {
                        int a = s[t], c = s[x];
                        bool up = (t & k) == 0;
                        if (up ? (a > c) : (a < c)) {
                            s[t] = c;
                            s[x] = a;
                        }
                    }
                }
                __syncthreads();
            }
        }
        // keep the first of each run of equal values, drop the sentinels, in order
        for (int base = 0; base < P; base += kThreads) {
            int t = base + tid;
            int v = t < P ? s[t] : kSentinel;
            int keep = (v != kSentinel && (t == 0 || s[t - 1] != v)) ? 1 : 0;
            int total;
            int pos = block_exclusive_scan(keep, &total, wave_sums);
            if (keep) out[running + pos] = v;
            running += total;
        }
    } else {
        // bit set: membership of each column, one range of kChunkCols columns at a time
        unsigned *bm = (unsigned *)s;
        for (int64_t lo = 0; lo < n; lo += kChunkCols) {
            for (int t = tid; t < kSortCap; t += kThreads) bm[t] = 0u;
            __syncthreads();
            for (int64_t t = tid; t < len; t += kThreads) {
                int64_t j = (int64_t)col[b + t] - lo;
                if (j >= 0 && j < kChunkCols) atomicOr(&bm[j >> 5], 1u << (j & 31));
            }
            if (tid == 0 && i >= lo && i < lo + kChunkCols) atomicOr(&bm[(i - lo) >> 5], 1u << ((i - lo) & 31));
            __syncthreads();
            for (int base = 0; base < kSortCap; base += kThreads) {
                unsigned wd = bm[base + tid];
                int total;
                int pos = block_exclusive_scan(__popc(wd), &total, wave_sums);
                int o = running + pos;
                while (wd) {
                    int bit = __ffs(wd) - 1;
                    out[o++] = (int)(lo + (int64_t)(base + tid) * 32 + bit);
                    wd &= wd - 1;
                }
                running += total;
            }
            __syncthreads();
        }
    }
    if (tid == 0) deg[i] = running;
}

// --------------------------------------------------------------------------------------------- scan int32 -> int64
constexpr int kScanItems = 4;
constexpr int kScanTile = kThreads * kScanItems;

__global__ __launch_bounds__(kThreads) void k_scan_tile_sums(int64_t n, const int32_t *__restrict__ in,
                                                             int64_t *__restrict__ blocksum) {
    __shared__ long long red[kThreads];
    int64_t base = (int64_t)blockIdx.x * kScanTile;
    long long s = 0;
    for (int k = 0; k < kScanItems; ++k) {
        int64_t p = base + (int64_t)threadIdx.x * kScanItems + k;
        if (p < n) s += in[p];
    }
    red[threadIdx.x] = s;
    __syncthreads();
    for (int d = kThreads / 2; d > 0; d >>= 1) {
        if (threadIdx.x < d) red[threadIdx.x] += red[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) blocksum[blockIdx.x] = red[0];
}

// One workgroup: blocksum[b] <- sum of blocksum[0..b) ; blocksum[nb] <- grand total.
__global__ __launch_bounds__(kThreads) void k_scan_block_sums(int64_t nb, int64_t *__restrict__ blocksum) {
    __shared__ long long tot[kThreads];
    __shared__ long long carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (int64_t base = 0; base < nb; base += kThreads) {
        int64_t p = base + threadIdx.x;
        long long v = p < nb ? blocksum[p] : 0;
        tot[threadIdx.x] = v;
        __syncthreads();
        // Hillis-Steele inclusive scan in LDS
        for (int d = 1; d < kThreads; d <<= 1) {
            long long add = threadIdx.x >= d ? tot[threadIdx.x - d] : 0;
            __syncthreads();
            tot[threadIdx.x] += add;
            __syncthreads();
        }
        long long c = carry;
        if (p < nb) blocksum[p] = c + tot[threadIdx.x] - v;
        __syncthreads();
        if (threadIdx.x == kThreads - 1) carry = c + tot[threadIdx.x];
        __syncthreads();
    }
    if (threadIdx.x == 0) blocksum[nb] = carry;
}

__global__ __launch_bounds__(kThreads) void k_scan_apply(int64_t n, const int32_t *__restrict__ in,
                                                         const int64_t *__restrict__ blocksum, int64_t nb,
                                                         int64_t *__restrict__ out /* n + 1 */) {
    __shared__ int wave_sums[4];
    int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    int v[kScanItems];
    int mine = 0;
    for (int k = 0; k < kScanItems; ++k) {
        v[k] = (base + k < n) ? in[base + k] : 0;
        mine += v[k];
    }
    int total;
    int pos = block_exclusive_scan(mine, &total, wave_sums);
    long long run = blocksum[blockIdx.x] + pos;
    for (int k = 0; k < kScanItems; ++k) {
        if (base + k < n) out[base + k] = run;
        run += v[k];
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) out[n] = blocksum[nb];
}

int exclusive_scan(int64_t n, const int32_t *in, int64_t *out, int64_t *blocksum, hipStream_t st) {
    int64_t nb = (n + kScanTile - 1) / kScanTile;
    k_scan_tile_sums<<<dim3((unsigned)nb), dim3(kThreads), 0, st>>>(n, in, blocksum);
    GCN_LAUNCH_CHECK();
    k_scan_block_sums<<<dim3(1), dim3(kThreads), 0, st>>>(nb, blocksum);
    GCN_LAUNCH_CHECK();
    k_scan_apply<<<dim3((unsigned)nb), dim3(kThreads), 0, st>>>(n, in, blocksum, nb, out);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

// --------------------------------------------------------------------------------------------- compaction, checks
// One wave per row: copy deg[i] columns from the scratch slot of row i to its final place.
__global__ __launch_bounds__(kThreads) void k_compact_rows(int64_t n, const int64_t *__restrict__ rowptr_in,
                                                           const int32_t *__restrict__ scratch,
                                                           const int64_t *__restrict__ rowptr,
                                                           int32_t *__restrict__ col, int32_t *flags) {
    int64_t i = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (i >= n) return;
    int lane = threadIdx.x & 63;
    const int32_t *src = scratch + rowptr_in[i] + i;
    int64_t o = rowptr[i];
    int64_t d = rowptr[i + 1] - o;
    for (int64_t t = lane; t < d; t += 64) col[o + t] = src[t];
    if (lane == 0) atomicMax(&flags[3], (int)d);
}

// One wave per row i: every column j of row i must have i in row j (binary search; rows are sorted).
__global__ __launch_bounds__(kThreads) void k_check_symmetric(int64_t n, const int64_t *__restrict__ rowptr,
                                                              const int32_t *__restrict__ col, int32_t *flags) {
    int64_t i = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (i >= n) return;
    int lane = threadIdx.x & 63;
    bool bad = false;
    for (int64_t p = rowptr[i] + lane; p < rowptr[i + 1]; p += 64) {
        int j = col[p];
        int64_t lo = rowptr[j], hi = rowptr[j + 1];
        while (lo < hi) {
            int64_t mid = (lo + hi) >> 1;
            if (col[mid] < (int)i) lo = mid + 1; else hi = mid;
        }
        if (lo >= rowptr[j + 1] || col[lo] != (int)i) bad = true;
    }
    if (bad) atomicOr(&flags[0], 4);
}

__global__ void k_dinv(int64_t n, const int32_t *__restrict__ deg, float *__restrict__ dinv) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dinv[i] = (float)(1.0 / sqrt((double)deg[i]));
}

// --------------------------------------------------------------------------------------------- schedule
__global__ void k_flag_classes(int64_t n, const int32_t *__restrict__ deg, int32_t *__restrict__ heavy,
                               int32_t *__restrict__ light) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int d = deg[i];
    heavy[i] = (d >= kHeavyDegree && d <= kSplitDegree) ? 1 : 0;
    light[i] = d < kHeavyDegree ? 1 : 0;
}

// Stable three-way partition: heavy rows keep their order in slots [0, n_heavy), light rows theirs after, split rows last.
__global__ void k_place_rows(int64_t n, const int32_t *__restrict__ heavy, const int32_t *__restrict__ light,
                             const int64_t *__restrict__ hpos, const int64_t *__restrict__ lpos,
                             int32_t *__restrict__ perm, int32_t *flags) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int64_t n_heavy = hpos[n], n_light = lpos[n];
    int64_t slot;
    if (heavy[i]) slot = hpos[i];
    else if (light[i]) slot = n_heavy + lpos[i];
    else slot = n_heavy + n_light + (i - hpos[i] - lpos[i]);
    perm[slot] = (int32_t)i;
    if (i == 0) {
        flags[4] = (int32_t)n_heavy;
        flags[5] = (int32_t)n_light;
    }
}

// row_start[x] = first row with at least x / kXcds of all entries before it (rowptr is that prefix sum)
__global__ void k_row_starts(int64_t n, const int64_t *__restrict__ rowptr, int32_t *__restrict__ row_start,
                             int by_entries) {
    const int x = threadIdx.x;
    if (x > kXcds) return;
    const int64_t total = rowptr[n];
    int64_t lo = 0, hi = n;
    if (x == kXcds) {
        lo = n;
    } else if (!by_entries) {
        const int64_t block = (n + kXcds - 1) / kXcds;
        lo = block * x < n ? block * x : n;
    } else {
        const int64_t target = total / kXcds * x + (total % kXcds) * x / kXcds;
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            if (rowptr[mid] < target) lo = mid + 1; else hi = mid;
        }
    }
    row_start[x] = (int32_t)lo;
}

// w[s] = entries of the heavy row in schedule slot s (0 for the other slots)
__global__ void k_heavy_weights(int64_t n, const int32_t *__restrict__ deg, const int32_t *__restrict__ perm,
                                const int32_t *__restrict__ flags, int32_t *__restrict__ w) {
    const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s < n) w[s] = s < flags[4] ? deg[perm[s]] : 0;
}
// before[s] = entries in the heavy slots before s; xcd_start[x] = first slot with at least x / kXcds of all of them
__global__ void k_xcd_starts(int64_t n, const int64_t *__restrict__ before, const int32_t *__restrict__ flags,
                             int32_t *__restrict__ xcd_start) {
    const int x = threadIdx.x;
    if (x > kXcds) return;
    const int64_t n_heavy = flags[4];
    const int64_t total = before[n];
    int64_t lo = 0, hi = n_heavy;
    if (x == kXcds) {
        lo = n_heavy;
    } else {
        const int64_t target = total / kXcds * x + (total % kXcds) * x / kXcds;
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            if (before[mid] < target) lo = mid + 1; else hi = mid;
        }
    }
    xcd_start[x] = (int32_t)lo;
}

// Chunks of the split rows: cnt[j] = number of chunks of split row j (0 past the last one) ...
__global__ void k_split_count(int64_t n, int64_t cap, const int32_t *__restrict__ deg, const int32_t *__restrict__ perm,
                              const int64_t *__restrict__ hpos, const int64_t *__restrict__ lpos,
                              int32_t *__restrict__ cnt) {
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= cap) return;
    const int64_t first = hpos[n] + lpos[n];
    cnt[j] = first + j < n ? (deg[perm[first + j]] + kChunk - 1) / kChunk : 0;
}
// ... and chunk_srow[c] = j for every chunk c of split row j
__global__ void k_split_fill(int64_t n, int64_t cap, const int64_t *__restrict__ hpos, const int64_t *__restrict__ lpos,
                             const int32_t *__restrict__ cnt, const int64_t *__restrict__ chunk_off,
                             int32_t *__restrict__ chunk_srow) {
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= cap || hpos[n] + lpos[n] + j >= n) return;
    for (int k = 0; k < cnt[j]; ++k) chunk_srow[chunk_off[j] + k] = (int32_t)j;
}

// One wave per row: lane b (0..kColBlocks) finds, by bisection in the sorted row, the offset of the first column
// that is >= b * block (block = ids per column range); lane kColBlocks gets the row length.
__global__ __launch_bounds__(kThreads) void k_segment_offsets(int64_t n, const int64_t *__restrict__ rowptr,
                                                              const int32_t *__restrict__ col, int64_t block,
                                                              int32_t *__restrict__ segoff) {
    const int64_t r = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (r >= n || lane > kColBlocks) return;
    const int64_t beg = rowptr[r], end = rowptr[r + 1];
    int64_t lo = beg, hi = end;
    if (lane < kColBlocks) {
        const int64_t bound = (int64_t)lane * block;
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            if ((int64_t)col[mid] < bound) lo = mid + 1; else hi = mid;
        }
    } else {
        lo = end;
    }
    segoff[r * (kColBlocks + 1) + lane] = (int32_t)(lo - beg);
}

// Phased schedule: which rows each wave of XCD x owns.  One workgroup per id range x: sorts the range's rows by
// degree (descending, ties by id) in LDS, then deals them to W waves in serpentine order, R per wave, so that every
// wave carries nearly the same number of entries: prow[(x * W + q) * R + j] = row (or -1).
constexpr int kMaxRangeRows = 8192;
__global__ __launch_bounds__(kThreads) void k_balance_rows(int64_t n, const int32_t *__restrict__ row_start,
                                                           const int32_t *__restrict__ deg, int W, int R,
                                                           int32_t *__restrict__ prow) {
    __shared__ unsigned long long key[kMaxRangeRows];
    const int x = blockIdx.x;
    const int64_t lo = row_start[x];
    const int64_t hi = row_start[x + 1] < n ? row_start[x + 1] : n;
    const int m = hi > lo ? (int)(hi - lo) : 0;
    int P = 2;
    while (P < m) P <<= 1;
    // ascending sort of (~degree, id): largest degree first, smaller id first among equals; padding sorts last
    for (int t = threadIdx.x; t < P; t += kThreads)
        key[t] = t < m ? (((unsigned long long)(0x7fffffffu - (unsigned)deg[lo + t])) << 32) | (unsigned)(lo + t)
                       : ~0ull;
    __syncthreads();
    for (int k = 2; k <= P; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = threadIdx.x; t < P; t += kThreads) {
                int y = t ^ j;
                if (y > t) {
                    unsigned long long a = key[t], c = key[y];
                    bool up = (t & k) == 0;
                    if (up ? (a > c) : (a < c)) {
                        key[t] = c;
                        key[y] = a;
                    }
                }
            }
            __syncthreads();
        }
    }
    for (int idx = threadIdx.x; idx < W * R; idx += kThreads) {
        const int q = idx / R, j = idx % R;
        const int rank = (j & 1) ? j * W + (W - 1 - q) : j * W + q;
        prow[((int64_t)x * W + q) * R + j] = rank < m ? (int32_t)(key[rank] & 0xffffffffu) : -1;
    }
}

__global__ void k_labels_mask(int64_t n, const int32_t *__restrict__ labels, const uint8_t *__restrict__ mask,
                              int32_t n_classes, int32_t *__restrict__ labels_out, uint8_t *__restrict__ mask_out,
                              int32_t *flags) {
    int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    bool in = false;
    if (v < n) {
        int32_t y = labels[v];
        if (y < 0 || y >= n_classes) atomicOr(&flags[1], 1);
        labels_out[v] = y;
        in = mask[v] != 0;
        mask_out[v] = in ? 1 : 0;
    }
    unsigned long long b = __ballot(in);
    if ((threadIdx.x & 63) == 0 && b) atomicAdd(&flags[2], __popcll(b));
}

inline unsigned blocks_for(int64_t items, int per_block) { return (unsigned)((items + per_block - 1) / per_block); }

}  // namespace

size_t scan_blocks(int64_t n) { return (size_t)((n + kScanTile - 1) / kScanTile) + 2; }

int exclusive_scan_i32(int64_t n, const int32_t *in, int64_t *out, int64_t *blocksum, hipStream_t st) {
    return exclusive_scan(n, in, out, blocksum, st);
}

int prep_validate(int64_t n, int64_t nnz_in, const int64_t *rowptr, const int32_t *col, int32_t *flags,
                  hipStream_t st) {
    k_validate_rowptr<<<dim3(blocks_for(n + 1, kThreads)), dim3(kThreads), 0, st>>>(n, nnz_in, rowptr, flags);
    GCN_LAUNCH_CHECK();
    if (nnz_in > 0) {
        k_validate_col<<<dim3(blocks_for(nnz_in, kThreads)), dim3(kThreads), 0, st>>>(n, nnz_in, col, flags);
        GCN_LAUNCH_CHECK();
    }
    return GCN_OK;
}

int prep_canonical(int64_t n, int64_t nnz_in, const int64_t *rowptr, const int32_t *col, PrepBuffers &pb,
                   hipStream_t st) {
    (void)nnz_in;
    k_canonical_rows<<<dim3((unsigned)n), dim3(kThreads), 0, st>>>(n, rowptr, col, pb.scratch, pb.deg);
    GCN_LAUNCH_CHECK();
    int rc = exclusive_scan(n, pb.deg, pb.rowptr, pb.blocksum, st);
    if (rc) return rc;
    k_compact_rows<<<dim3(blocks_for(n, kThreads / 64)), dim3(kThreads), 0, st>>>(n, rowptr, pb.scratch, pb.rowptr,
                                                                                   pb.col, pb.flags);
    GCN_LAUNCH_CHECK();
    k_check_symmetric<<<dim3(blocks_for(n, kThreads / 64)), dim3(kThreads), 0, st>>>(n, pb.rowptr, pb.col, pb.flags);
    GCN_LAUNCH_CHECK();
    k_dinv<<<dim3(blocks_for(n, kThreads)), dim3(kThreads), 0, st>>>(n, pb.deg, pb.dinv);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int prep_schedule(int64_t n, PrepBuffers &pb, hipStream_t st) {
    int32_t *light = pb.scratch;   // n flags; the canonicalisation is done with this buffer by now
    k_flag_classes<<<dim3(blocks_for(n, kThreads)), dim3(kThreads), 0, st>>>(n, pb.deg, pb.heavy, light);
    GCN_LAUNCH_CHECK();
    int rc = exclusive_scan(n, pb.heavy, pb.hpos, pb.blocksum, st);
    if (rc) return rc;
    rc = exclusive_scan(n, light, pb.lpos, pb.blocksum, st);
    if (rc) return rc;
    k_place_rows<<<dim3(blocks_for(n, kThreads)), dim3(kThreads), 0, st>>>(n, pb.heavy, light, pb.hpos, pb.lpos, pb.perm,
                                                                            pb.flags);
    GCN_LAUNCH_CHECK();
    k_split_count<<<dim3(blocks_for(pb.split_cap, kThreads)), dim3(kThreads), 0, st>>>(n, pb.split_cap, pb.deg, pb.perm,
                                                                                        pb.hpos, pb.lpos, pb.split_cnt);
    GCN_LAUNCH_CHECK();
    rc = exclusive_scan(pb.split_cap, pb.split_cnt, pb.chunk_off, pb.blocksum, st);
    if (rc) return rc;
    k_split_fill<<<dim3(blocks_for(pb.split_cap, kThreads)), dim3(kThreads), 0, st>>>(n, pb.split_cap, pb.hpos, pb.lpos,
                                                                                       pb.split_cnt, pb.chunk_off,
                                                                                       pb.chunk_srow);
    GCN_LAUNCH_CHECK();
    // the heavy rows' shares of the XCDs (pb.heavy and pb.hpos are free again)
    k_heavy_weights<<<dim3(blocks_for(n, kThreads)), dim3(kThreads), 0, st>>>(n, pb.deg, pb.perm, pb.flags, pb.heavy);
    GCN_LAUNCH_CHECK();
    rc = exclusive_scan(n, pb.heavy, pb.hpos, pb.blocksum, st);
    if (rc) return rc;
    k_xcd_starts<<<dim3(1), dim3(64), 0, st>>>(n, pb.hpos, pb.flags, pb.xcd_start);
    GCN_LAUNCH_CHECK();
    k_row_starts<<<dim3(1), dim3(64), 0, st>>>(n, pb.rowptr, pb.row_start, (int)tunable("phased_balance", 1));
    GCN_LAUNCH_CHECK();
    if (pb.segoff) {   // only graphs small enough for the phased schedule carry the table
        const int64_t block = (n + kColBlocks - 1) / kColBlocks;
        k_segment_offsets<<<dim3(blocks_for(n, kThreads / 64)), dim3(kThreads), 0, st>>>(n, pb.rowptr, pb.col, block,
                                                                                          pb.segoff);
        GCN_LAUNCH_CHECK();
    }
    return GCN_OK;
}

namespace {

// One wave per row: the entries whose column c has keep[c] != 0, in their order.
//   WRITE = false: deg_out[r] = how many;  WRITE = true: col_out filled from rowptr_out[r] on
template <bool WRITE>
__global__ __launch_bounds__(kThreads) void k_keep_columns(int64_t n, const int64_t *__restrict__ rowptr,
                                                           const int32_t *__restrict__ col,
                                                           const uint8_t *__restrict__ keep,
                                                           int32_t *__restrict__ deg_out,
                                                           const int64_t *__restrict__ rowptr_out,
                                                           int32_t *__restrict__ col_out) {
    const int64_t r = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (r >= n) return;
    const int lane = threadIdx.x & 63;
    const int64_t beg = rowptr[r], end = rowptr[r + 1];
    const int64_t out0 = WRITE ? rowptr_out[r] : 0;
    int count = 0;
    for (int64_t e0 = beg; e0 < end; e0 += 64) {
        const int64_t e = e0 + lane;
        int c = 0;
        bool kept = false;
        if (e < end) {
            c = col[e];
            kept = keep[c] != 0;
        }
        const unsigned long long b = __ballot(kept);
        if (WRITE && kept) col_out[out0 + count + __popcll(b & ((1ull << lane) - 1ull))] = c;
        count += __popcll(b);
    }
    if (!WRITE && lane == 0) deg_out[r] = count;
}

}  // namespace

int prep_keep_columns(int64_t n, const PrepBuffers &src, const uint8_t *keep, PrepBuffers &dst, hipStream_t st) {
    k_keep_columns<false><<<dim3(blocks_for(n, kThreads / 64)), dim3(kThreads), 0, st>>>(n, src.rowptr, src.col, keep,
                                                                                          dst.deg, nullptr, nullptr);
    GCN_LAUNCH_CHECK();
    int rc = exclusive_scan_i32(n, dst.deg, dst.rowptr, dst.blocksum, st);
    if (rc) return rc;
    k_keep_columns<true><<<dim3(blocks_for(n, kThreads / 64)), dim3(kThreads), 0, st>>>(n, src.rowptr, src.col, keep,
                                                                                         nullptr, dst.rowptr, dst.col);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int prep_balance_rows(int64_t n, const int32_t *deg, const int32_t *row_start, int W, int R, int32_t *prow,
                      hipStream_t st) {
    if ((int64_t)W * R > kMaxRangeRows) {
        set_error("phased schedule: more than %d rows per range", kMaxRangeRows);
        return GCN_EINVAL;
    }
    k_balance_rows<<<dim3(kXcds), dim3(kThreads), 0, st>>>(n, row_start, deg, W, R, prow);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int prep_labels_mask(int64_t n, const int32_t *labels, const uint8_t *mask, int32_t n_classes, int32_t *labels_out,
                     uint8_t *mask_out, int32_t *flags, hipStream_t st) {
    k_labels_mask<<<dim3(blocks_for(n, kThreads)), dim3(kThreads), 0, st>>>(n, labels, mask, n_classes, labels_out,
                                                                            mask_out, flags);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

}  // namespace gcn

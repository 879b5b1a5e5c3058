// Subgraph approximation: the augmented partition P_o[p] of Algorithm 1 ("breadth-first random sampling
// of vertices", Section 3.1), then the induced subgraph, i.e. every edge without both ends in P_o[p] is
// dropped (Section 4).  All integer work, set semantics, results independent of thread timing.
//
// For every other partition op, level 1 is the set of op's vertices adjacent to p, level k + 1 the
// set of op's vertices adjacent to level k and not seen before.  Levels are taken whole while they fit
// into nts = floor(O N_p / (M - 1)); from the first level that does not fit, the missing number of
// vertices is drawn: those with the smallest key(v) = mix(mix(seed) ^ v) (mix = SplitMix64's output
// function, a bijection, hence no ties).  The k-th smallest key is found by bisection over the 64-bit
// key range with a counting kernel; all partitions that need a draw at the same level search together.
// The breadth-first expansion runs for all other partitions at once, one level per launch.
#include <vector>

#include "common.hpp"

namespace gcn {

namespace {

constexpr int kThreads = 256;
constexpr int kMaxParts = 1024;

__device__ inline uint64_t mix64a(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

uint64_t host_mix(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

inline unsigned blocks_for(int64_t items, int per_block) { return (unsigned)((items + per_block - 1) / per_block); }

__global__ void k_check_parts(int64_t n, const int32_t *__restrict__ part, int32_t n_parts, int32_t p,
                              int32_t *__restrict__ level, int32_t *__restrict__ sel, int32_t *misc) {
    int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    bool local = false;
    if (v < n) {
        const int32_t q = part[v];
        if (q < 0 || q >= n_parts) atomicOr(&misc[0], 1);
        local = q == p;
        level[v] = 0;
        sel[v] = 0;
    }
    const unsigned long long b = __ballot(local);
    if ((threadIdx.x & 63) == 0 && b) atomicAdd(&misc[1], __popcll(b));
}

// One wave per vertex v of the current frontier: mark its unseen neighbours in still-active partitions.
// k == 1: the frontier is partition p itself and it reaches into every other partition;
// k  > 1: the frontier is level k - 1 and it stays inside its own partition.
__global__ __launch_bounds__(kThreads) void k_expand(int64_t n, const int64_t *__restrict__ rowptr,
                                                     const int32_t *__restrict__ col,
                                                     const int32_t *__restrict__ part, int32_t p, int32_t k,
                                                     const int32_t *__restrict__ active,
                                                     int32_t *__restrict__ level, int32_t *__restrict__ count) {
    const int64_t v = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (v >= n) return;
    const int lane = threadIdx.x & 63;
    const int32_t pv = part[v];
    if (k == 1) {
        if (pv != p) return;
    } else {
        if (pv == p || level[v] != k - 1 || !active[pv]) return;
    }
    for (int64_t e = rowptr[v] + lane; e < rowptr[v + 1]; e += 64) {
        const int32_t u = col[e];
        const int32_t pu = part[u];
        if (pu == p || !active[pu]) continue;
        if (k > 1 && pu != pv) continue;
        if (atomicCAS(&level[u], 0, k) == 0) atomicAdd(&count[pu], 1);
    }
}

// mode[op]: 0 nothing, 1 take the whole level, 2 take the vertices with key <= threshold[op]
__global__ void k_take(int64_t n, const int32_t *__restrict__ part, const int32_t *__restrict__ level, int32_t k,
                       const int32_t *__restrict__ mode, const uint64_t *__restrict__ threshold, uint64_t seed_key,
                       int32_t *__restrict__ sel) {
    int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= n || level[u] != k) return;
    const int32_t op = part[u];
    const int32_t md = mode[op];
    if (md == 1) sel[u] = 1;
    else if (md == 2 && mix64a(seed_key ^ (uint64_t)u) <= threshold[op]) sel[u] = 1;
}

// count_le[op] += number of level-k vertices of op (mode 2 only) with key <= threshold[op]
__global__ void k_count_le(int64_t n, const int32_t *__restrict__ part, const int32_t *__restrict__ level, int32_t k,
                           const int32_t *__restrict__ mode, const uint64_t *__restrict__ threshold,
                           uint64_t seed_key, int32_t *__restrict__ count_le) {
    int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= n || level[u] != k) return;
    const int32_t op = part[u];
    if (mode[op] == 2 && mix64a(seed_key ^ (uint64_t)u) <= threshold[op]) atomicAdd(&count_le[op], 1);
}

__global__ void k_flags(int64_t n, const int32_t *__restrict__ part, int32_t p, const int32_t *__restrict__ sel,
                        int32_t *__restrict__ flag_local, int32_t *__restrict__ flag_sel) {
    int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= n) return;
    flag_local[v] = part[v] == p ? 1 : 0;
    flag_sel[v] = sel[v] ? 1 : 0;
}

__global__ void k_new_ids(int64_t n, const int32_t *__restrict__ flag_local, const int32_t *__restrict__ flag_sel,
                          const int64_t *__restrict__ pos_local, const int64_t *__restrict__ pos_sel,
                          int32_t *__restrict__ new_id, int32_t *__restrict__ vertices) {
    int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= n) return;
    int64_t id = -1;
    if (flag_local[v]) id = pos_local[v];
    else if (flag_sel[v]) id = pos_local[n] + pos_sel[v];
    new_id[v] = (int32_t)id;
    if (id >= 0) vertices[id] = (int32_t)v;
}

// One wave per kept vertex.  FILL == false: count the neighbours that are kept too.  FILL == true: write
// their new ids, in the order of the input row.
template <bool FILL>
__global__ __launch_bounds__(kThreads) void k_induced(int64_t n_out, const int32_t *__restrict__ vertices,
                                                      const int64_t *__restrict__ rowptr,
                                                      const int32_t *__restrict__ col,
                                                      const int32_t *__restrict__ new_id,
                                                      int32_t *__restrict__ row_len,
                                                      const int64_t *__restrict__ rowptr_out,
                                                      int32_t *__restrict__ col_out) {
    const int64_t i = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (i >= n_out) return;
    const int lane = threadIdx.x & 63;
    const int64_t v = vertices[i];
    const int64_t beg = rowptr[v], end = rowptr[v + 1];
    int64_t running = FILL ? rowptr_out[i] : 0;
    for (int64_t base = beg; base < end; base += 64) {
        const int64_t e = base + lane;
        int32_t id = -1;
        if (e < end) id = new_id[col[e]];
        const unsigned long long keep = __ballot(id >= 0);
        if (FILL && id >= 0) {
            const int before = __popcll(keep & ((1ull << lane) - 1ull));
            col_out[running + before] = id;
        }
        running += __popcll(keep);
    }
    if (!FILL && lane == 0) row_len[i] = (int32_t)running;
}

__global__ void k_gather_rows(const uint32_t *__restrict__ src, size_t row_words, const int32_t *__restrict__ idx,
                              int64_t n_idx, uint32_t *__restrict__ dst) {
    size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (size_t)n_idx * row_words) return;
    const size_t r = t / row_words, c = t - r * row_words;
    dst[t] = src[(size_t)idx[r] * row_words + c];
}

struct Buffers {
    int32_t *level, *sel, *flag_local, *flag_sel, *new_id, *row_len, *misc, *active, *count, *mode, *count_le;
    int64_t *pos_local, *pos_sel, *blocksum;
    uint64_t *threshold;
};

void carve(Carver &c, Buffers &b, int64_t n) {
    b.level = c.take<int32_t>(n);
    b.sel = c.take<int32_t>(n);
    b.flag_local = c.take<int32_t>(n);
    b.flag_sel = c.take<int32_t>(n);
    b.new_id = c.take<int32_t>(n);
    b.row_len = c.take<int32_t>(n);
    b.pos_local = c.take<int64_t>(n + 1);
    b.pos_sel = c.take<int64_t>(n + 1);
    b.blocksum = c.take<int64_t>(scan_blocks(n));
    b.misc = c.take<int32_t>(16);
    b.active = c.take<int32_t>(kMaxParts);
    b.count = c.take<int32_t>(kMaxParts);
    b.mode = c.take<int32_t>(kMaxParts);
    b.count_le = c.take<int32_t>(kMaxParts);
    b.threshold = c.take<uint64_t>(kMaxParts);
}

}  // namespace

size_t augment_workspace_bytes(int64_t n) {
    Carver c(nullptr);
    Buffers b;
    carve(c, b, n);
    return c.bytes();
}

int gather_rows(const void *src, size_t row_bytes, const int32_t *idx, int64_t n_idx, void *dst, hipStream_t st) {
    if (n_idx <= 0) return GCN_OK;
    if (row_bytes == 0 || row_bytes % 4 != 0) {
        set_error("gather_rows: row size must be a positive multiple of 4 bytes");
        return GCN_EINVAL;
    }
    const size_t words = row_bytes / 4;
    k_gather_rows<<<dim3(blocks_for((int64_t)(n_idx * words), kThreads)), dim3(kThreads), 0, st>>>(
        (const uint32_t *)src, words, idx, n_idx, (uint32_t *)dst);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int augment_partition(int64_t n, const int64_t *rowptr, const int32_t *col, const int32_t *part, int32_t n_parts,
                      int32_t p, double overlap, uint64_t seed, void *workspace, int64_t *n_out, int64_t *n_local_out,
                      int64_t *nnz_out, int32_t *vertices, int64_t *rowptr_out, int32_t *col_out, hipStream_t st) {
    Carver c(workspace);
    Buffers b;
    carve(c, b, n);
    const int M = n_parts;
    const uint64_t seed_key = host_mix(seed);
    std::vector<int32_t> h_active(M, 1), h_count(M, 0), h_mode(M, 0), h_le(M, 0);
    std::vector<int64_t> need(M, 0);
    std::vector<uint64_t> lo(M, 0), hi(M, 0), thr(M, 0);
    int32_t misc[16];

    int rc = fill_zero(b.misc, 16 * sizeof(int32_t), st);
    if (rc) return rc;
    k_check_parts<<<dim3(blocks_for(n, kThreads)), dim3(kThreads), 0, st>>>(n, part, n_parts, p, b.level, b.sel, b.misc);
    GCN_LAUNCH_CHECK();
    GCN_HIP(hipMemcpyAsync(misc, b.misc, sizeof(misc), hipMemcpyDeviceToHost, st));
    GCN_HIP(hipStreamSynchronize(st));
    if (misc[0]) {
        set_error("gcn_augment_partition: a partition id is outside [0, %d)", n_parts);
        return GCN_EINVAL;
    }
    const int64_t n_p = misc[1];
    const int64_t nts = M > 1 ? (int64_t)std::floor(overlap * (double)n_p / (double)(M - 1)) : 0;
    for (int op = 0; op < M; ++op) {
        need[op] = nts;
        h_active[op] = (op != p && nts > 0) ? 1 : 0;
    }

    for (int32_t k = 1; k <= n; ++k) {   // a level adds at least one vertex or ends a partition's search
        bool any = false;
        for (int op = 0; op < M; ++op) any = any || h_active[op];
        if (!any) break;
        GCN_HIP(hipMemcpyAsync(b.active, h_active.data(), M * sizeof(int32_t), hipMemcpyHostToDevice, st));
        rc = fill_zero(b.count, (size_t)M * sizeof(int32_t), st);
        if (rc) return rc;
        k_expand<<<dim3(blocks_for(n, kThreads / 64)), dim3(kThreads), 0, st>>>(n, rowptr, col, part, p, k, b.active,
                                                                              b.level, b.count);
        GCN_LAUNCH_CHECK();
        GCN_HIP(hipMemcpyAsync(h_count.data(), b.count, M * sizeof(int32_t), hipMemcpyDeviceToHost, st));
        GCN_HIP(hipStreamSynchronize(st));
        bool draw = false;
        for (int op = 0; op < M; ++op) {
            h_mode[op] = 0;
            if (!h_active[op]) continue;
            const int64_t cnt = h_count[op];
            if (cnt == 0) {
                h_active[op] = 0;
            } else if (cnt < need[op]) {
                h_mode[op] = 1;
                need[op] -= cnt;
            } else if (cnt == need[op]) {
                h_mode[op] = 1;
                need[op] = 0;
                h_active[op] = 0;
            } else {
                h_mode[op] = 2;
                draw = true;
                lo[op] = 0;
                hi[op] = ~0ull;
                h_active[op] = 0;
            }
        }
        GCN_HIP(hipMemcpyAsync(b.mode, h_mode.data(), M * sizeof(int32_t), hipMemcpyHostToDevice, st));
        if (draw) {
            // smallest threshold with at least need[op] keys at or below it; keys are distinct, so exactly need[op]
            for (int it = 0; it < 64; ++it) {
                for (int op = 0; op < M; ++op) thr[op] = lo[op] + (hi[op] - lo[op]) / 2;
                GCN_HIP(hipMemcpyAsync(b.threshold, thr.data(), M * sizeof(uint64_t), hipMemcpyHostToDevice, st));
                rc = fill_zero(b.count_le, (size_t)M * sizeof(int32_t), st);
                if (rc) return rc;
                k_count_le<<<dim3(blocks_for(n, kThreads)), dim3(kThreads), 0, st>>>(n, part, b.level, k, b.mode,
                                                                                    b.threshold, seed_key, b.count_le);
                GCN_LAUNCH_CHECK();
                GCN_HIP(hipMemcpyAsync(h_le.data(), b.count_le, M * sizeof(int32_t), hipMemcpyDeviceToHost, st));
                GCN_HIP(hipStreamSynchronize(st));
                for (int op = 0; op < M; ++op) {
                    if (h_mode[op] != 2 || lo[op] >= hi[op]) continue;
                    if ((int64_t)h_le[op] >= need[op]) hi[op] = thr[op];
                    else lo[op] = thr[op] + 1;
                }
            }
            for (int op = 0; op < M; ++op) thr[op] = lo[op];
            GCN_HIP(hipMemcpyAsync(b.threshold, thr.data(), M * sizeof(uint64_t), hipMemcpyHostToDevice, st));
        }
        k_take<<<dim3(blocks_for(n, kThreads)), dim3(kThreads), 0, st>>>(n, part, b.level, k, b.mode, b.threshold,
                                                                        seed_key, b.sel);
        GCN_LAUNCH_CHECK();
        GCN_HIP(hipStreamSynchronize(st));   // the host vectors above are reused in the next round
    }

    // new ids: partition p in ascending order, then the sampled vertices in ascending order
    k_flags<<<dim3(blocks_for(n, kThreads)), dim3(kThreads), 0, st>>>(n, part, p, b.sel, b.flag_local, b.flag_sel);
    GCN_LAUNCH_CHECK();
    rc = exclusive_scan_i32(n, b.flag_local, b.pos_local, b.blocksum, st);
    if (rc) return rc;
    rc = exclusive_scan_i32(n, b.flag_sel, b.pos_sel, b.blocksum, st);
    if (rc) return rc;
    k_new_ids<<<dim3(blocks_for(n, kThreads)), dim3(kThreads), 0, st>>>(n, b.flag_local, b.flag_sel, b.pos_local,
                                                                       b.pos_sel, b.new_id, vertices);
    GCN_LAUNCH_CHECK();
    int64_t ends[2];
    GCN_HIP(hipMemcpyAsync(&ends[0], b.pos_local + n, sizeof(int64_t), hipMemcpyDeviceToHost, st));
    GCN_HIP(hipMemcpyAsync(&ends[1], b.pos_sel + n, sizeof(int64_t), hipMemcpyDeviceToHost, st));
    GCN_HIP(hipStreamSynchronize(st));
    const int64_t total = ends[0] + ends[1];
    if (total > 0) {
        k_induced<false><<<dim3(blocks_for(total, kThreads / 64)), dim3(kThreads), 0, st>>>(
            total, vertices, rowptr, col, b.new_id, b.row_len, nullptr, nullptr);
        GCN_LAUNCH_CHECK();
        rc = exclusive_scan_i32(total, b.row_len, rowptr_out, b.blocksum, st);
        if (rc) return rc;
        k_induced<true><<<dim3(blocks_for(total, kThreads / 64)), dim3(kThreads), 0, st>>>(
            total, vertices, rowptr, col, b.new_id, nullptr, rowptr_out, col_out);
        GCN_LAUNCH_CHECK();
    }
    int64_t nnz = 0;
    if (total > 0) GCN_HIP(hipMemcpyAsync(&nnz, rowptr_out + total, sizeof(int64_t), hipMemcpyDeviceToHost, st));
    GCN_HIP(hipStreamSynchronize(st));
    *n_out = total;
    *n_local_out = ends[0];
    *nnz_out = nnz;
    return GCN_OK;
}

}  // namespace gcn

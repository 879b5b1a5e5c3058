// Aggregation  Z = A_hat T  (the sparse product of Section 4.1's layer rule; the nnz(A) F term of the
// cost model in Section 5.4), also used unchanged for the backward pass because A_hat is symmetric.
//
// The factor d_j^-1/2 of A_hat_ij = d_i^-1/2 d_j^-1/2 is already folded into the rows of the input
// (its producer scales row j once), so a row of the output is a plain sum of gathered input rows
// times d_i^-1/2.  No value array is read: 4 bytes of column index per nonzero.  Rows are walked in
// schedule order; each scheduled row is padded to a multiple of kRowPad entries with column n, an
// all-zero input row, so the inner loop has no tail.
//
// Work split: a group of LPR lanes owns one output row; each lane carries one float4 of the row
// (LPR * 4 >= leading dimension).  A wave therefore works on 64 / LPR rows at once.  Column indices
// are fetched LPR at a time, one per lane (coalesced), and handed round the group by cross-lane
// reads; feature rows are fetched as 16-byte loads, a whole row per group per load instruction.
#include "common.hpp"

namespace gcn {

namespace {

constexpr int kThreads = 256;

__device__ inline uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

struct Epi {
    int kind;
    int width;
    uint32_t drop_threshold;
    float keep_scale;
    uint64_t drop_key;
};

__device__ inline float finish(float v, const Epi &ep, int64_t row, int c) {
    if (ep.kind == kEpiRelu) {
        v = v > 0.0f ? v : 0.0f;
        if (ep.drop_threshold != 0u) {
            uint64_t e = (uint64_t)row * (uint64_t)ep.width + (uint64_t)c;
            uint64_t h = mix64(ep.drop_key + e * 0x9E3779B97F4A7C15ull);
            v = ((uint32_t)(h >> 32) >= ep.drop_threshold) ? v * ep.keep_scale : 0.0f;
        }
    }
    return v;
}

template <int LPR, int U>
__global__ __launch_bounds__(kThreads) void k_spmm_group(const int64_t *__restrict__ rowptr_p,
                                                         const int32_t *__restrict__ col_p,
                                                         const int32_t *__restrict__ perm,
                                                         const float *__restrict__ dinv, int64_t n,
                                                         const float *__restrict__ t, int ld_t,
                                                         float *__restrict__ out, int ld_out, int nblocks, Epi ep) {
    static_assert(kRowPad % U == 0, "rows are padded to a multiple of the unroll");
    static_assert(LPR % U == 0, "one index fetch feeds a whole number of unrolled steps");
    constexpr int GPW = 64 / LPR;                 // rows per wave
    constexpr int RPB = (kThreads / 64) * GPW;    // rows per workgroup
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane / LPR, sub = lane % LPR;
    // consecutive workgroup ids land on different XCDs; give each XCD one contiguous range of rows
    const int per_xcd = (nblocks + kXcds - 1) / kXcds;
    const int blk = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
    if (blk >= nblocks) return;
    const int64_t s = (int64_t)blk * RPB + wave * GPW + grp;
    const bool live = s < n;
    const bool lane_on = sub * 4 < ld_t;
    int64_t beg = 0, end = 0;
    int r = 0;
    if (live) {
        beg = rowptr_p[s];
        end = rowptr_p[s + 1];
        r = perm[s];
    }
    const float4 *tv = reinterpret_cast<const float4 *>(t) + sub;
    const int ld4 = ld_t >> 2;
    float4 acc0 = make_float4(0.f, 0.f, 0.f, 0.f);
    float4 acc1 = make_float4(0.f, 0.f, 0.f, 0.f);
    int nxt = (beg + sub < end) ? col_p[beg + sub] : (int)n;
    for (int64_t e = beg; e < end; e += LPR) {
        const int mine = nxt;
        const int cnt = (end - e) < LPR ? (int)(end - e) : LPR;
        const int64_t e2 = e + LPR + sub;
        nxt = (e2 < end) ? col_p[e2] : (int)n;
        for (int k = 0; k < cnt; k += U) {
            int c[U];
            float4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) c[u] = __shfl(mine, grp * LPR + k + u, 64);
#pragma unroll
            for (int u = 0; u < U; ++u)
                v[u] = lane_on ? tv[(int64_t)c[u] * ld4] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int u = 0; u < U; u += 2) {
                acc0.x += v[u].x; acc0.y += v[u].y; acc0.z += v[u].z; acc0.w += v[u].w;
                acc1.x += v[u + 1].x; acc1.y += v[u + 1].y; acc1.z += v[u + 1].z; acc1.w += v[u + 1].w;
            }
        }
    }
    if (live && sub * 4 < ld_out) {
        const float d = dinv[r];
        const int c0 = sub * 4;
        float4 o;
        o.x = finish((acc0.x + acc1.x) * d, ep, r, c0 + 0);
        o.y = finish((acc0.y + acc1.y) * d, ep, r, c0 + 1);
        o.z = finish((acc0.z + acc1.z) * d, ep, r, c0 + 2);
        o.w = finish((acc0.w + acc1.w) * d, ep, r, c0 + 3);
        reinterpret_cast<float4 *>(out + (int64_t)r * ld_out)[sub] = o;
    }
}

template <int LPR>
int launch_group(const SpmmArgs &a, hipStream_t st) {
    constexpr int RPB = (kThreads / 64) * (64 / LPR);
    const int nblocks = (int)((a.n + RPB - 1) / RPB);
    const int grid = (nblocks + kXcds - 1) / kXcds * kXcds;
    Epi ep{a.epilogue, a.width, a.drop_threshold, a.keep_scale, a.drop_key};
    k_spmm_group<LPR, (LPR < 8 ? LPR : 8)><<<dim3(grid), dim3(kThreads), 0, st>>>(a.rowptr_p, a.col_p, a.perm, a.dinv, a.n, a.t,
                                                                 a.ld_t, a.out, a.ld_out, nblocks, ep);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

}  // namespace

int spmm_launch(const SpmmArgs &a, hipStream_t st) {
    if (a.n <= 0) return GCN_OK;
    if (a.ld_t % 4 != 0 || a.ld_out % 4 != 0 || a.ld_out > a.ld_t || a.ld_t > 256) {
        set_error("aggregation: unsupported leading dimensions %d / %d", a.ld_t, a.ld_out);
        return GCN_EINVAL;
    }
    timing_begin(a.width, st);
    int rc;
    const int vecs = a.ld_t / 4;
    if (vecs <= 4) rc = launch_group<4>(a, st);
    else if (vecs <= 8) rc = launch_group<8>(a, st);
    else if (vecs <= 16) rc = launch_group<16>(a, st);
    else if (vecs <= 32) rc = launch_group<32>(a, st);
    else rc = launch_group<64>(a, st);
    timing_end(st);
    return rc;
}

}  // namespace gcn

// Dense products of the training step on the matrix cores (fp32 MFMA 32x32x2, fp32 accumulate):
//   nn  T = D^-1/2 (H W)                      feature transform of Section 4.1's layer rule
//   nt  dZ_prev = D^-1/2 ((G W^T) * [H > 0])  input gradient with the ReLU gate
//   tn  dW = H^T G                            weight gradient, reduced over all vertices
// (the N F^2 term of the cost model in Section 5.4).  The D^-1/2 row scale belongs to the
// aggregation that consumes the result: A_hat_ij = d_i^-1/2 d_j^-1/2, and the d_j^-1/2 half is
// applied here, once per row, instead of once per nonzero there.
//
// One workgroup = 4 waves.  A wave owns a 32-row strip and TN column tiles of 32; per k-step of 16
// the operands pass through LDS.  v_mfma_f32_32x32x2f32 takes, per lane l, A[l % 32][l / 32] and
// B[l / 32][l % 32] and keeps D[8 (v / 4) + 4 (l / 32) + v % 4][l % 32] in accumulator register v.
// Which two k of the 16 a lane pair feeds at each step is free (a sum is a sum): lane half h feeds
// k = 8 h + s at step s, so the A fragment is two 16-byte LDS reads.
#include "common.hpp"
#include "epilogue.hpp"
#include "plane_sink.hpp"

namespace gcn {

namespace {

constexpr int kThreads = 256;
constexpr int BK = 16;
constexpr int kApad = 4;

typedef float f32x16 __attribute__((ext_vector_type(16)));

enum Mode { kNN = 0, kNT = 1, kTN = 2 };

struct GemmArgs {
    const float *a;
    int lda;
    const float *b;
    int ldb;
    float *c;
    int ldc;
    int64_t M;      // rows of the output (nn, nt) / rows reduced over (tn)
    int K;          // shared dimension (nn, nt) / output rows (tn)
    int N;          // output columns
    const float *rowscale;
    const float *gate;
    int ldg;
    float scale;
    int64_t rows_per_split;  // tn
    Activation act;          // nn: applied after the row scale
    int k_per_split;         // nn: 0 = the whole shared dimension in one workgroup; else blockIdx.y takes this many k
                             // and writes its own partial matrix (M x ldc, one after the other at c)
    PlaneSink sink;          // nn without split, nt: the output once more, as the tile product's operand planes
};

template <int MODE, int WM, int WN, int TN>
__global__ __launch_bounds__(kThreads) void k_gemm(GemmArgs g) {
    constexpr int BM = 32 * WM;
    constexpr int BN = 32 * TN * WN;
    static_assert(WM * WN == kThreads / 64, "four waves");
    // nn/nt: As[m][k] (k contiguous, padded);  tn: As[k][m] (m contiguous)
    constexpr int kAsFloats = (MODE == kTN) ? BK * BM : BM * (BK + kApad);
    __shared__ __attribute__((aligned(16))) float As[kAsFloats];
    // nn/tn: Bs[k][n] as loaded;  nt: the operand arrives [n][k] and is turned round on the way in, four 4-byte
    // stores per float4: rows padded by 4 floats so that the four k-quarters of a column land in different banks
    // (unpadded they hit one bank: 54 % of the kernel's LDS cycles were conflicts)
    constexpr int BNP = (MODE == kNT) ? BN + 4 : BN;
    __shared__ __attribute__((aligned(16))) float Bs[BK * BNP];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int h = lane >> 5, l32 = lane & 31;

    int64_t m0;     // first output row of this workgroup
    int n0;         // first output column
    int64_t kbeg, kend;
    if (MODE == kTN) {
        const int mtiles = (g.K + BM - 1) / BM;
        m0 = (int64_t)(blockIdx.x % mtiles) * BM;
        n0 = (blockIdx.x / mtiles) * BN;
        kbeg = (int64_t)blockIdx.y * g.rows_per_split;
        kend = kbeg + g.rows_per_split < g.M ? kbeg + g.rows_per_split : g.M;
    } else {
        const int ntiles = (g.N + BN - 1) / BN;
        m0 = (int64_t)(blockIdx.x / ntiles) * BM;
        n0 = (blockIdx.x % ntiles) * BN;
        kbeg = 0;
        kend = g.K;
        if (MODE == kNN && g.k_per_split > 0) {
            kbeg = (int64_t)blockIdx.y * g.k_per_split;
            kend = kbeg + g.k_per_split < g.K ? kbeg + g.k_per_split : g.K;
        }
    }

    f32x16 acc[TN];
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;

    constexpr int A_VECS = BM * BK / 4, B_VECS = BK * BN / 4;
    constexpr int A_PER = (A_VECS + kThreads - 1) / kThreads, B_PER = (B_VECS + kThreads - 1) / kThreads;
    float4 ra[A_PER], rb[B_PER];

    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int i = 0; i < A_PER; ++i) {
            const int idx = tid + i * kThreads;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (idx < A_VECS) {
                if (MODE == kTN) {
                    const int k = idx / (BM / 4), m4 = idx % (BM / 4);
                    const int64_t row = k0 + k;
                    const int64_t colm = m0 + m4 * 4;
                    if (row < kend && colm < g.lda) v = *reinterpret_cast<const float4 *>(g.a + row * g.lda + colm);
                } else {
                    const int m = idx / (BK / 4), kq = idx % (BK / 4);
                    const int64_t row = m0 + m;
                    if (row < g.M) v = *reinterpret_cast<const float4 *>(g.a + row * g.lda + k0 + kq * 4);
                }
            }
            ra[i] = v;
        }
#pragma unroll
        for (int i = 0; i < B_PER; ++i) {
            const int idx = tid + i * kThreads;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (idx < B_VECS) {
                if (MODE == kNT) {
                    const int nn = idx / (BK / 4), kq = idx % (BK / 4);
                    const int row = n0 + nn;
                    if (row < g.N) v = *reinterpret_cast<const float4 *>(g.b + (int64_t)row * g.ldb + k0 + kq * 4);
                } else {
                    const int k = idx / (BN / 4), n4 = idx % (BN / 4);
                    const int64_t row = k0 + k;
                    const int coln = n0 + n4 * 4;
                    if (row < kend && coln < g.ldb) v = *reinterpret_cast<const float4 *>(g.b + row * g.ldb + coln);
                }
            }
            rb[i] = v;
        }
    };

    auto stash = [&]() {
#pragma unroll
        for (int i = 0; i < A_PER; ++i) {
            const int idx = tid + i * kThreads;
            if (idx < A_VECS) {
                if (MODE == kTN) {
                    *reinterpret_cast<float4 *>(&As[idx * 4]) = ra[i];               // [k][m], same order as idx
                } else {
                    const int m = idx / (BK / 4), kq = idx % (BK / 4);
                    *reinterpret_cast<float4 *>(&As[m * (BK + kApad) + kq * 4]) = ra[i];
                }
            }
        }
#pragma unroll
        for (int i = 0; i < B_PER; ++i) {
            const int idx = tid + i * kThreads;
            if (idx < B_VECS) {
                if (MODE == kNT) {
                    const int nn = idx / (BK / 4), kq = idx % (BK / 4);
                    Bs[(kq * 4 + 0) * BNP + nn] = rb[i].x;
                    Bs[(kq * 4 + 1) * BNP + nn] = rb[i].y;
                    Bs[(kq * 4 + 2) * BNP + nn] = rb[i].z;
                    Bs[(kq * 4 + 3) * BNP + nn] = rb[i].w;
                } else {
                    *reinterpret_cast<float4 *>(&Bs[idx * 4]) = rb[i];               // [k][n], same order as idx
                }
            }
        }
    };

    if (kbeg < kend) fetch(kbeg);
    for (int64_t k0 = kbeg; k0 < kend; k0 += BK) {
        __syncthreads();           // everyone is done reading the previous tiles
        stash();
        __syncthreads();
        if (k0 + BK < kend) fetch(k0 + BK);
        float af[8];
        if (MODE == kTN) {
#pragma unroll
            for (int s = 0; s < 8; ++s) af[s] = As[(h * 8 + s) * BM + wm * 32 + l32];
        } else {
            const float4 lo = *reinterpret_cast<const float4 *>(&As[(wm * 32 + l32) * (BK + kApad) + h * 8]);
            const float4 hi = *reinterpret_cast<const float4 *>(&As[(wm * 32 + l32) * (BK + kApad) + h * 8 + 4]);
            af[0] = lo.x; af[1] = lo.y; af[2] = lo.z; af[3] = lo.w;
            af[4] = hi.x; af[5] = hi.y; af[6] = hi.z; af[7] = hi.w;
        }
#pragma unroll
        for (int t = 0; t < TN; ++t) {
            const int cb = (wn * TN + t) * 32 + l32;
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const float bf = Bs[(h * 8 + s) * BNP + cb];
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[s], bf, acc[t], 0, 0, 0);
            }
        }
    }

    // epilogue
    const int64_t out_rows = (MODE == kTN) ? (int64_t)g.K : g.M;
    float *cbase = g.c;
    if (MODE == kTN) cbase += (int64_t)blockIdx.y * (int64_t)g.K * g.ldc;   // this split's partial matrix
    if (MODE == kNN && g.k_per_split > 0) cbase += (int64_t)blockIdx.y * g.M * g.ldc;
    const bool to_sink = MODE != kTN && g.sink.planes && !(MODE == kNN && g.k_per_split > 0);
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        const int col = n0 + (wn * TN + t) * 32 + l32;
        float xs[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int64_t row = m0 + wm * 32 + 8 * (v / 4) + 4 * h + (v % 4);
            float x = 0.0f;
            if (row < out_rows && col < g.ldc) {
                x = acc[t][v];
                if (MODE == kNN) {
                    if (g.rowscale) x *= g.rowscale[row];
                    x = activate(x, g.act, row, col);
                } else if (MODE == kNT) {
                    const float gt = g.gate ? g.gate[row * g.ldg + col] : 1.0f;
                    x = gt > 0.0f ? x * g.scale : 0.0f;
                    if (g.rowscale) x *= g.rowscale[row];
                }
                cbase[row * g.ldc + col] = x;
            }
            xs[v] = x;
        }
        if (to_sink) sink_store(g.sink, m0 + wm * 32, col, h, xs);
    }
}

// c[i] = sum over the splits of partials[split][i], in a fixed order: the splits are cut into kReduceGroups
// consecutive runs, eight threads add one run each in ascending order (one float4 of the output per thread, four
// loads in flight), and the runs' sums are added in ascending order.  A single thread per output would wait
// through a hundred dependent round trips.
constexpr int kReduceGroups = 8;
constexpr int kReduceOutputs = 256 / kReduceGroups;   // float4 outputs per workgroup

__global__ __launch_bounds__(256) void k_reduce_partials(const float4 *__restrict__ partials, int splits,
                                                         size_t count4, float4 *__restrict__ c) {
    __shared__ float4 sm[kReduceGroups][kReduceOutputs];
    const int o = threadIdx.x % kReduceOutputs, grp = threadIdx.x / kReduceOutputs;
    const size_t i = (size_t)blockIdx.x * kReduceOutputs + o;
    const int per = (splits + kReduceGroups - 1) / kReduceGroups;
    const int beg = grp * per, end = beg + per < splits ? beg + per : splits;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < count4) {
        int p = beg;
        for (; p + 4 <= end; p += 4) {
            float4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = partials[(size_t)(p + u) * count4 + i];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                s.x += v[u].x;
                s.y += v[u].y;
                s.z += v[u].z;
                s.w += v[u].w;
            }
        }
        for (; p < end; ++p) {
            const float4 v = partials[(size_t)p * count4 + i];
            s.x += v.x;
            s.y += v.y;
            s.z += v.z;
            s.w += v.w;
        }
    }
    sm[grp][o] = s;
    __syncthreads();
    if (grp == 0 && i < count4) {
        float4 t = sm[0][o];
#pragma unroll
        for (int q = 1; q < kReduceGroups; ++q) {
            t.x += sm[q][o].x;
            t.y += sm[q][o].y;
            t.z += sm[q][o].z;
            t.w += sm[q][o].w;
        }
        c[i] = t;
    }
}

// as k_reduce_partials, then max(., 0) when relu is set
__global__ void k_reduce_partials_relu(const float4 *__restrict__ partials, int splits, size_t count4,
                                       float4 *__restrict__ c, int relu) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count4) return;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int p = 0; p < splits; ++p) {
        const float4 v = partials[(size_t)p * count4 + i];
        s.x += v.x;
        s.y += v.y;
        s.z += v.z;
        s.w += v.w;
    }
    if (relu) {
        s.x = s.x > 0.f ? s.x : 0.f;
        s.y = s.y > 0.f ? s.y : 0.f;
        s.z = s.z > 0.f ? s.z : 0.f;
        s.w = s.w > 0.f ? s.w : 0.f;
    }
    c[i] = s;
}

template <int MODE>
int launch_rows(GemmArgs &g, hipStream_t st) {   // nn, nt
    if (g.N > 64) {
        const int ntiles = (g.N + 127) / 128;
        const int64_t tiles64 = (g.M + 63) / 64 * ntiles;
        if (tiles64 < 4 * 256 && g.K <= 128) {
            // fewer than four workgroups per CU: half-height tiles double the waves that hide each other's waits
            // (over a long shared dimension the second read of B costs as much as that gains)
            const unsigned grid = (unsigned)((g.M + 31) / 32) * ntiles;
            k_gemm<MODE, 1, 4, 1><<<dim3(grid), dim3(kThreads), 0, st>>>(g);
        } else {
            k_gemm<MODE, 2, 2, 2><<<dim3((unsigned)tiles64), dim3(kThreads), 0, st>>>(g);
        }
    } else if (g.N > 32) {
        const unsigned grid = (unsigned)((g.M + 127) / 128);
        if (grid < 4 * 256)   // as above
            k_gemm<MODE, 2, 2, 1><<<dim3((unsigned)((g.M + 63) / 64)), dim3(kThreads), 0, st>>>(g);
        else
            k_gemm<MODE, 4, 1, 2><<<dim3(grid), dim3(kThreads), 0, st>>>(g);
    } else {
        const unsigned grid = (unsigned)((g.M + 127) / 128);
        k_gemm<MODE, 4, 1, 1><<<dim3(grid), dim3(kThreads), 0, st>>>(g);
    }
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int tn_splits(int64_t rows, int M, int N) {
    const int mtiles = (M + 127) / 128;
    const int bn = N > 64 ? 128 : (N > 32 ? 64 : 32);
    const int ntiles = (N + bn - 1) / bn;
    int splits = 512 / (mtiles * ntiles);
    if (splits < 1) splits = 1;
    const int64_t max_by_rows = (rows + 4 * BK - 1) / (4 * BK);   // at least 64 rows per split
    if (splits > max_by_rows) splits = (int)max_by_rows;
    if (splits < 1) splits = 1;
    return splits;
}

bool check_ld(int lda, int ldb, int ldc) { return lda % 16 == 0 && ldb % 16 == 0 && ldc % 16 == 0; }

}  // namespace

int gemm_nn(const float *a, int lda, const float *b, int ldb, float *c, int ldc, int64_t M, int K, int N,
            const float *rowscale, const Activation *act, hipStream_t st, const PlaneSink *sink) {
    if (M <= 0) return GCN_OK;
    if (!check_ld(lda, ldb, ldc) || K % BK != 0 || K > lda || N > ldb) {
        set_error("gemm_nn: bad shape M=%lld K=%d N=%d lda=%d ldb=%d ldc=%d", (long long)M, K, N, lda, ldb, ldc);
        return GCN_EINVAL;
    }
    GemmArgs g{a, lda, b, ldb, c, ldc, M, K, N, rowscale, nullptr, 0, 1.0f, 0, act ? *act : Activation{kActNone, 0, 0u, 1.0f, 0ull}, 0,
               sink ? *sink : PlaneSink{nullptr, 0, 0}};
    return launch_rows<kNN>(g, st);
}

// For few rows: the shared dimension is split over blockIdx.y so that the chip fills, the partial matrices are
// added in ascending order (and passed through max(., 0) if relu is set).
int nn_splits(int64_t M, int K, int N) {
    const int64_t tiles = ((M + 63) / 64) * ((N + 127) / 128);
    int splits = (int)(512 / (tiles > 0 ? tiles : 1));
    const int max_by_k = K / (4 * BK) > 0 ? K / (4 * BK) : 1;    // at least 64 of the shared dimension per split
    if (splits > max_by_k) splits = max_by_k;
    return splits < 1 ? 1 : splits;
}

size_t gemm_nn_splitk_partial_floats(int64_t M, int K, int N) {
    return (size_t)nn_splits(M, K, N) * (size_t)M * (size_t)padded_width(N);
}

int gemm_nn_splitk(const float *a, int lda, const float *b, int ldb, float *c, int ldc, int64_t M, int K, int N,
                   bool relu, float *partials, size_t partial_floats, hipStream_t st) {
    if (M <= 0) return GCN_OK;
    if (!check_ld(lda, ldb, ldc) || K % BK != 0 || K > lda || N > ldb || N > 128 * 65535) {
        set_error("gemm_nn_splitk: bad shape M=%lld K=%d N=%d lda=%d ldb=%d ldc=%d", (long long)M, K, N, lda, ldb, ldc);
        return GCN_EINVAL;
    }
    const int splits = nn_splits(M, K, N);
    if ((size_t)splits * (size_t)M * (size_t)ldc > partial_floats) {
        set_error("gemm_nn_splitk: partial buffer too small");
        return GCN_EWORKSPACE;
    }
    int per = (K + splits - 1) / splits;
    per = (per + BK - 1) / BK * BK;
    GemmArgs g{a, lda, b, ldb, partials, ldc, M, K, N, nullptr, nullptr, 0, 1.0f, 0, Activation{kActNone, 0, 0u, 1.0f, 0ull}, per, PlaneSink{nullptr, 0, 0}};
    const int ntiles = (N + 127) / 128;
    const unsigned gx = (unsigned)((M + 63) / 64) * ntiles;
    k_gemm<kNN, 2, 2, 2><<<dim3(gx, (unsigned)splits), dim3(kThreads), 0, st>>>(g);
    GCN_LAUNCH_CHECK();
    const size_t count4 = (size_t)M * (size_t)ldc / 4;
    k_reduce_partials_relu<<<dim3((unsigned)((count4 + 255) / 256)), dim3(256), 0, st>>>(
        reinterpret_cast<const float4 *>(partials), splits, count4, reinterpret_cast<float4 *>(c), relu ? 1 : 0);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int gemm_nt(const float *a, int lda, const float *b, int ldb, float *c, int ldc, int64_t M, int K, int N,
            const float *rowscale, const float *gate, int ldg, float scale, hipStream_t st, const PlaneSink *sink) {
    if (M <= 0) return GCN_OK;
    if (!check_ld(lda, ldb, ldc) || K % BK != 0 || K > lda || K > ldb || (gate && ldg < ldc)) {
        set_error("gemm_nt: bad shape M=%lld K=%d N=%d lda=%d ldb=%d ldc=%d", (long long)M, K, N, lda, ldb, ldc);
        return GCN_EINVAL;
    }
    GemmArgs g{a, lda, b, ldb, c, ldc, M, K, N, rowscale, gate, ldg, scale, 0, Activation{kActNone, 0, 0u, 1.0f, 0ull}, 0,
               sink ? *sink : PlaneSink{nullptr, 0, 0}};
    return launch_rows<kNT>(g, st);
}

size_t gemm_tn_partial_floats(int64_t rows, int M, int N) {
    (void)N;
    // the partial matrices use the output's leading dimension, which is at most padded_width(N)
    return (size_t)tn_splits(rows, M, N) * (size_t)M * (size_t)padded_width(N);
}

int gemm_tn(const float *a, int lda, const float *b, int ldb, float *c, int ldc, int64_t rows, int M, int N,
            float *partials, size_t partial_floats, hipStream_t st) {
    if (!check_ld(lda, ldb, ldc) || M > lda || N > ldb || N > ldc) {
        set_error("gemm_tn: bad shape rows=%lld M=%d N=%d lda=%d ldb=%d ldc=%d", (long long)rows, M, N, lda, ldb, ldc);
        return GCN_EINVAL;
    }
    const int splits = tn_splits(rows, M, N);
    if ((size_t)splits * (size_t)M * (size_t)ldc > partial_floats) {
        set_error("gemm_tn: partial buffer too small");
        return GCN_EWORKSPACE;
    }
    int64_t per = (rows + splits - 1) / splits;
    per = (per + BK - 1) / BK * BK;
    GemmArgs g{a, lda, b, ldb, partials, ldc, rows, M, N, nullptr, nullptr, 0, 1.0f, per, Activation{kActNone, 0, 0u, 1.0f, 0ull}, 0,
               PlaneSink{nullptr, 0, 0}};
    const int mtiles = (M + 127) / 128;
    if (N > 64) {
        const int ntiles = (N + 127) / 128;
        k_gemm<kTN, 4, 1, 4><<<dim3(mtiles * ntiles, splits), dim3(kThreads), 0, st>>>(g);
    } else if (N > 32) {
        k_gemm<kTN, 4, 1, 2><<<dim3(mtiles, splits), dim3(kThreads), 0, st>>>(g);
    } else {
        k_gemm<kTN, 4, 1, 1><<<dim3(mtiles, splits), dim3(kThreads), 0, st>>>(g);
    }
    GCN_LAUNCH_CHECK();
    return reduce_partials(partials, splits, (size_t)M * (size_t)ldc, c, st);
}

int reduce_partials(const float *partials, int splits, size_t count, float *c, hipStream_t st) {
    const size_t count4 = count / 4;   // leading dimensions are multiples of 16
    k_reduce_partials<<<dim3((unsigned)((count4 + kReduceOutputs - 1) / kReduceOutputs)), dim3(256), 0, st>>>(
        reinterpret_cast<const float4 *>(partials), splits, count4, reinterpret_cast<float4 *>(c));
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

}  // namespace gcn

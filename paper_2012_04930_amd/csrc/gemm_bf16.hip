// The three dense products of the training step for bfloat16 storage: bf16 operands on the matrix
// cores (v_mfma_f32_32x32x16_bf16), float32 accumulation.
//   nn  T = D^-1/2 (H W)                      a = H [M x K],  b = W^T stored [N x K]      -> bf16
//   nt  dZ_prev = D^-1/2 ((G W^T) * [H > 0])  a = G [M x K],  b = W   stored [N x K]      -> bf16
//   tn  dW = H^T G                            a = H [rows x M], b = G [rows x N]          -> float32 partials
// (feature transform and gradients of Section 4.1's layer rule; the N F^2 term of Section 5.4.)
//
// The instruction takes 8 consecutive-k bf16 per lane for both operands: lane l feeds row/column
// l % 32 and the k-octet l / 32 of a 16-deep step.  Both operands therefore sit in LDS with k
// contiguous ([m][k] and [n][k], rows padded to 40 elements so the 16-byte fragment reads spread
// over all banks).  nn and nt read their operands that way from memory already (the weights are
// kept in both orientations); tn has the reduction index as the slow one in memory, so its loader
// turns 4 x 8 blocks round in registers before the LDS store.
#include "common.hpp"
#include "dtypes.hpp"
#include "epilogue.hpp"

namespace gcn {

namespace {

constexpr int kThreads = 256;
constexpr int BK = 32;
constexpr int LDS_LD = BK + 8;   // bf16 elements per LDS row (80 bytes)

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // 16 bytes in flight (a plain vector: stays in registers)

enum Mode { kNN = 0, kNT = 1, kTN = 2 };

struct Args {
    const bf16_t *a;
    int lda;
    const bf16_t *b;
    int ldb;
    void *c;
    int ldc;
    int64_t M;      // output rows (nn, nt) / rows reduced over (tn)
    int K;          // shared dimension (nn, nt) / output rows (tn)
    int N;          // output columns
    const float *rowscale;
    const bf16_t *gate;
    int ldg;
    float scale;
    int64_t rows_per_split;
    Activation act;   // nn: applied after the row scale
};

__device__ inline uint32_t pack_lo(uint32_t a, uint32_t b) { return (a & 0xffffu) | (b << 16); }
__device__ inline uint32_t pack_hi(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xffff0000u); }

template <int MODE, int WM, int WN, int TN>
__global__ __launch_bounds__(kThreads) void k_gemm_bf16(Args g) {
    constexpr int BM = 32 * WM;
    constexpr int BN = 32 * TN * WN;
    static_assert(WM * WN == kThreads / 64, "four waves");
    // LDS: the two operand tiles during the product; afterwards (nn, nt) the same bytes hold the output tile as
    // bfloat16, rows C_LD apart, so that it leaves in 16-byte pieces along the rows
    constexpr int C_LD = BN + 8;
    constexpr int kStageBytes = (BM + BN) * LDS_LD * 2;
    constexpr int kOutBytes = MODE == kTN ? 0 : BM * C_LD * 2;
    __shared__ __attribute__((aligned(16))) unsigned char smem[kStageBytes > kOutBytes ? kStageBytes : kOutBytes];
    bf16_t *const As = reinterpret_cast<bf16_t *>(smem);
    bf16_t *const Bs = As + BM * LDS_LD;
    bf16_t *const Cs = reinterpret_cast<bf16_t *>(smem);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int h = lane >> 5, l32 = lane & 31;

    int64_t m0, kbeg, kend;
    int n0;
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
    }

    f32x16 acc[TN];
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;

    // ---- nn / nt staging: 16-byte vectors along k
    constexpr int A_VECS = BM * BK / 8, B_VECS = BN * BK / 8;
    constexpr int A_PER = (A_VECS + kThreads - 1) / kThreads, B_PER = (B_VECS + kThreads - 1) / kThreads;
    // ---- tn staging: units of 4 k-rows x 8 columns, A units first, then B units; at most one per thread
    constexpr int A_UNITS = (BK / 4) * (BM / 8), B_UNITS = (BK / 4) * (BN / 8);
    static_assert(MODE != kTN || A_UNITS + B_UNITS <= kThreads, "one transposing unit per thread");
    uint4 ra[MODE == kTN ? 4 : 1];                                    // tn: the four rows of a unit
    u32x4 va[MODE == kTN ? 1 : A_PER], vb[MODE == kTN ? 1 : B_PER];   // nn, nt

    auto fetch = [&](int64_t k0) {
        if (MODE == kTN) {
            const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
            for (int j = 0; j < 4; ++j) ra[j] = zero;
            if (tid < A_UNITS + B_UNITS) {
                const bool isA = tid < A_UNITS;
                const int u = isA ? tid : tid - A_UNITS;
                const int kgroup = u % (BK / 4), chunk = u / (BK / 4);
                const bf16_t *src = isA ? g.a : g.b;
                const int ld = isA ? g.lda : g.ldb;
                const int64_t c0 = (isA ? m0 : (int64_t)n0) + chunk * 8;
                if (c0 < ld) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int64_t row = k0 + kgroup * 4 + j;
                        if (row < kend) ra[j] = *reinterpret_cast<const uint4 *>(src + row * ld + c0);
                    }
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < A_PER; ++i) {
                const int idx = tid + i * kThreads;
                u32x4 v = {0u, 0u, 0u, 0u};
                if (idx < A_VECS) {
                    const int m = idx / (BK / 8), kq = idx % (BK / 8);
                    const int64_t row = m0 + m;
                    const int64_t k = k0 + kq * 8;
                    if (row < g.M && k < kend) v = *reinterpret_cast<const u32x4 *>(g.a + row * g.lda + k);
                }
                va[i] = v;
            }
#pragma unroll
            for (int i = 0; i < B_PER; ++i) {
                const int idx = tid + i * kThreads;
                u32x4 v = {0u, 0u, 0u, 0u};
                if (idx < B_VECS) {
                    const int nn = idx / (BK / 8), kq = idx % (BK / 8);
                    const int row = n0 + nn;
                    const int64_t k = k0 + kq * 8;
                    if (row < g.N && k < kend) v = *reinterpret_cast<const u32x4 *>(g.b + (int64_t)row * g.ldb + k);
                }
                vb[i] = v;
            }
        }
    };

    auto stash = [&]() {
        if (MODE == kTN) {
            if (tid < A_UNITS + B_UNITS) {
                const bool isA = tid < A_UNITS;
                const int u = isA ? tid : tid - A_UNITS;
                const int kgroup = u % (BK / 4), chunk = u / (BK / 4);
                bf16_t *dst = (isA ? As : Bs) + (chunk * 8) * LDS_LD + kgroup * 4;
                // ra[j] holds row j: 8 columns in 4 words; column i of rows 0..3 -> one 8-byte LDS store
                const uint32_t w[4][4] = {{ra[0].x, ra[0].y, ra[0].z, ra[0].w},
                                          {ra[1].x, ra[1].y, ra[1].z, ra[1].w},
                                          {ra[2].x, ra[2].y, ra[2].z, ra[2].w},
                                          {ra[3].x, ra[3].y, ra[3].z, ra[3].w}};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint2 even, odd;   // columns 2q and 2q + 1
                    even.x = pack_lo(w[0][q], w[1][q]);
                    even.y = pack_lo(w[2][q], w[3][q]);
                    odd.x = pack_hi(w[0][q], w[1][q]);
                    odd.y = pack_hi(w[2][q], w[3][q]);
                    *reinterpret_cast<uint2 *>(dst + (2 * q) * LDS_LD) = even;
                    *reinterpret_cast<uint2 *>(dst + (2 * q + 1) * LDS_LD) = odd;
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < A_PER; ++i) {
                const int idx = tid + i * kThreads;
                if (idx < A_VECS) {
                    const int m = idx / (BK / 8), kq = idx % (BK / 8);
                    *reinterpret_cast<u32x4 *>(&As[m * LDS_LD + kq * 8]) = va[i];
                }
            }
#pragma unroll
            for (int i = 0; i < B_PER; ++i) {
                const int idx = tid + i * kThreads;
                if (idx < B_VECS) {
                    const int nn = idx / (BK / 8), kq = idx % (BK / 8);
                    *reinterpret_cast<u32x4 *>(&Bs[nn * LDS_LD + kq * 8]) = vb[i];
                }
            }
        }
    };

    if (kbeg < kend) fetch(kbeg);
    for (int64_t k0 = kbeg; k0 < kend; k0 += BK) {
        __syncthreads();
        stash();
        __syncthreads();
        if (k0 + BK < kend) fetch(k0 + BK);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const bf16x8 af = *reinterpret_cast<const bf16x8 *>(&As[(wm * 32 + l32) * LDS_LD + ks * 16 + h * 8]);
#pragma unroll
            for (int t = 0; t < TN; ++t) {
                const bf16x8 bfr =
                    *reinterpret_cast<const bf16x8 *>(&Bs[((wn * TN + t) * 32 + l32) * LDS_LD + ks * 16 + h * 8]);
                // nn, nt: the operands change places, so the instruction forms the transposed tile and a lane ends up
                // with four consecutive columns of ONE output row per register quad (see the epilogue below)
                acc[t] = MODE == kTN ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfr, acc[t], 0, 0, 0)
                                     : __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr, af, acc[t], 0, 0, 0);
            }
        }
    }

    if (MODE == kTN) {
        float *cb = static_cast<float *>(g.c) + (int64_t)blockIdx.y * (int64_t)g.K * g.ldc;   // this split's partial matrix
#pragma unroll
        for (int t = 0; t < TN; ++t) {
            const int col = n0 + (wn * TN + t) * 32 + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = m0 + wm * 32 + 8 * (v / 4) + 4 * h + (v % 4);
                if (row < (int64_t)g.K && col < g.ldc) cb[row * g.ldc + col] = acc[t][v];
            }
        }
        return;
    }

    // nn, nt.  With the operands in their usual places a lane would hold one column of 16 rows: 2-byte stores and
    // gate loads, one row scale and one float -> bfloat16 conversion per element, and the kernel is bound by
    // those vector instructions, not by the matrix pipes or memory.  With the operands swapped a lane holds, of
    // output row wm * 32 + l32, the columns 8 q + 4 h + 0..3 of each 32-column tile in registers 4 q .. 4 q + 3: one
    // row scale per lane, and four values at a time to gate, convert and store as 8 bytes.  The tile goes through
    // LDS (the bytes the operand tiles used): the gate tile comes in and the finished tile leaves in 16-byte pieces
    // along the rows, a whole row of the tile per 4 to 16 lanes.
    constexpr int ROW_VECS = BN / 8, TILE_VECS = BM * ROW_VECS, PER = TILE_VECS / kThreads;
    static_assert(TILE_VECS % kThreads == 0, "whole passes");
    __syncthreads();   // every wave has read its last fragments: the operand tiles may be overwritten
    if (MODE == kNT && g.gate) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int idx = tid + i * kThreads;
            const int r = idx / ROW_VECS, c = (idx % ROW_VECS) * 8;
            const int64_t row = m0 + r;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (row < g.M && n0 + c < g.ldc) v = *reinterpret_cast<const uint4 *>(g.gate + row * g.ldg + n0 + c);
            *reinterpret_cast<uint4 *>(&Cs[r * C_LD + c]) = v;
        }
        __syncthreads();
    }
    {
        const int rl = wm * 32 + l32;
        const int64_t row = m0 + rl;
        const bool live = row < g.M;
        const float rs = (live && g.rowscale) ? g.rowscale[row] : 1.0f;
        const bool relu = g.act.kind == kActRelu, drop = relu && g.act.drop_threshold != 0u;
#pragma unroll
        for (int t = 0; t < TN; ++t) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int cl = (wn * TN + t) * 32 + 8 * q + 4 * h;
                bf16_t *const spot = &Cs[rl * C_LD + cl];   // (this thread alone touches these four elements)
                float x[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) x[i] = acc[t][4 * q + i];
                if (MODE == kNT) {
                    if (g.gate) {
                        const uint2 gw = *reinterpret_cast<const uint2 *>(spot);
                        // a bfloat16 is positive when it is neither zero nor negative: sign clear, rest non-zero
                        const uint32_t e[4] = {gw.x & 0xffffu, gw.x >> 16, gw.y & 0xffffu, gw.y >> 16};
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float gt = __uint_as_float(e[i] << 16);
                            x[i] = gt > 0.0f ? x[i] * g.scale : 0.0f;
                        }
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i) x[i] *= g.scale;
                    }
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    x[i] *= rs;
                    if (MODE == kNN && relu) x[i] = x[i] > 0.0f ? x[i] : 0.0f;
                    if (MODE == kNN && drop && live) x[i] = activate(x[i], g.act, row, n0 + cl + i);   // (keeps or zeroes)
                }
                store_elems<4>(spot, x);   // 8 bytes
            }
        }
    }
    __syncthreads();
    bf16_t *const c = static_cast<bf16_t *>(g.c);
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int idx = tid + i * kThreads;
        const int r = idx / ROW_VECS, cc = (idx % ROW_VECS) * 8;
        const int64_t row = m0 + r;
        if (row < g.M && n0 + cc < g.ldc)
            *reinterpret_cast<uint4 *>(c + row * g.ldc + n0 + cc) = *reinterpret_cast<const uint4 *>(&Cs[r * C_LD + cc]);
    }
}

template <int MODE>
int launch_rows(Args &g, hipStream_t st) {
    if (g.N > 64) {
        const int ntiles = (g.N + 127) / 128;
        const unsigned grid = (unsigned)((g.M + 63) / 64) * ntiles;
        k_gemm_bf16<MODE, 2, 2, 2><<<dim3(grid), dim3(kThreads), 0, st>>>(g);
    } else if (g.N > 32) {
        k_gemm_bf16<MODE, 4, 1, 2><<<dim3((unsigned)((g.M + 127) / 128)), dim3(kThreads), 0, st>>>(g);
    } else {
        k_gemm_bf16<MODE, 4, 1, 1><<<dim3((unsigned)((g.M + 127) / 128)), dim3(kThreads), 0, st>>>(g);
    }
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

bool ok_ld(int lda, int ldb, int ldc) { return lda % 16 == 0 && ldb % 16 == 0 && ldc % 16 == 0; }

}  // namespace

int gemm_bf16_nn(const void *a, int lda, const void *bt, int ldb, void *c, int ldc, int64_t M, int K, int N,
                 const float *rowscale, const Activation *act, hipStream_t st) {
    if (M <= 0) return GCN_OK;
    if (!ok_ld(lda, ldb, ldc) || K % 16 != 0 || K > lda || K > ldb) {
        set_error("gemm_bf16_nn: bad shape M=%lld K=%d N=%d lda=%d ldb=%d ldc=%d", (long long)M, K, N, lda, ldb, ldc);
        return GCN_EINVAL;
    }
    Args g{(const bf16_t *)a, lda, (const bf16_t *)bt, ldb, c, ldc, M, K, N, rowscale, nullptr, 0, 1.0f, 0,
           act ? *act : Activation{kActNone, 0, 0u, 1.0f, 0ull}};
    return launch_rows<kNN>(g, st);
}

int gemm_bf16_nt(const void *a, int lda, const void *b, int ldb, void *c, int ldc, int64_t M, int K, int N,
                 const float *rowscale, const void *gate, int ldg, float scale, hipStream_t st) {
    if (M <= 0) return GCN_OK;
    if (!ok_ld(lda, ldb, ldc) || K % 16 != 0 || K > lda || K > ldb || (gate && ldg < ldc)) {
        set_error("gemm_bf16_nt: bad shape M=%lld K=%d N=%d lda=%d ldb=%d ldc=%d", (long long)M, K, N, lda, ldb, ldc);
        return GCN_EINVAL;
    }
    Args g{(const bf16_t *)a, lda, (const bf16_t *)b, ldb, c, ldc, M, K, N, rowscale, (const bf16_t *)gate, ldg, scale, 0,
           Activation{kActNone, 0, 0u, 1.0f, 0ull}};
    return launch_rows<kNT>(g, st);
}

int gemm_bf16_tn_splits(int64_t rows, int M, int N) {
    const int mtiles = (M + 127) / 128;
    const int bn = N > 64 ? 128 : (N > 32 ? 64 : 32);
    const int ntiles = (N + bn - 1) / bn;
    int splits = 1024 / (mtiles * ntiles);
    const int64_t max_by_rows = (rows + 8 * BK - 1) / (8 * BK);   // at least 256 rows per split
    if (splits > max_by_rows) splits = (int)max_by_rows;
    if (splits < 1) splits = 1;
    return splits;
}

size_t gemm_bf16_tn_partial_floats(int64_t rows, int M, int N) {
    return (size_t)gemm_bf16_tn_splits(rows, M, N) * (size_t)M * (size_t)padded_width(N);
}

int gemm_bf16_tn_partials(const void *a, int lda, const void *b, int ldb, int ldc, int64_t rows, int M, int N,
                          float *partials, size_t partial_floats, int *splits_out, hipStream_t st) {
    if (!ok_ld(lda, ldb, ldc) || M > lda || N > ldb || N > ldc) {
        set_error("gemm_bf16_tn: bad shape rows=%lld M=%d N=%d lda=%d ldb=%d ldc=%d", (long long)rows, M, N, lda, ldb,
                  ldc);
        return GCN_EINVAL;
    }
    const int splits = gemm_bf16_tn_splits(rows, M, N);
    if ((size_t)splits * (size_t)M * (size_t)ldc > partial_floats) {
        set_error("gemm_bf16_tn: partial buffer too small");
        return GCN_EWORKSPACE;
    }
    int64_t per = (rows + splits - 1) / splits;
    per = (per + BK - 1) / BK * BK;
    Args g{(const bf16_t *)a, lda, (const bf16_t *)b, ldb, partials, ldc, rows, M, N, nullptr, nullptr, 0, 1.0f, per,
           Activation{kActNone, 0, 0u, 1.0f, 0ull}};
    const int mtiles = (M + 127) / 128;
    if (N > 64) {
        const int ntiles = (N + 127) / 128;
        k_gemm_bf16<kTN, 4, 1, 4><<<dim3(mtiles * ntiles, splits), dim3(kThreads), 0, st>>>(g);
    } else if (N > 32) {
        k_gemm_bf16<kTN, 4, 1, 2><<<dim3(mtiles, splits), dim3(kThreads), 0, st>>>(g);
    } else {
        k_gemm_bf16<kTN, 4, 1, 1><<<dim3(mtiles, splits), dim3(kThreads), 0, st>>>(g);
    }
    GCN_LAUNCH_CHECK();
    *splits_out = splits;
    return GCN_OK;
}

}  // namespace gcn

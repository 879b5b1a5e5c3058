// Float32 dense product on the bfloat16 matrix instruction, for the large product of the first layer (feature
// transform H W of Section 4.1's layer rule; the N F^2 term of Section 5.4).
//
// Each operand is kept as three bfloat16 planes whose sum is the float32 value exactly (bf16_split.hpp).  With
// a = a0 + a1 + a2 and b = b0 + b1 + b2 the product is the sum of nine plane products; the three with i + j > 2
// are below 2^-23 |a| |b| and are left out, the other six run on v_mfma_f32_32x32x16_bf16 with float32
// accumulation.  Six bfloat16 steps of depth 16 cost 6 x 8 passes for what the float32 instruction (depth 2,
// 16 passes) needs 8 x 16 passes for.
//
// The product:  c [M x N] = a [M x K] b^T  (b has N rows of length K);  T = D^-1/2 (X W) has a = X [n x f] and
// b = W^T [d x f].
// The weight gradient of the same layer (dW = H^T G of the backward pass) is the same kernel's second form: a = the
// packed transpose [f x n], the shared index is the vertices, and the right operand G [n x d] is not packed per call
// (its transpose would be the long operand, read again by every row tile, and packing it costs a pass per epoch:
// measured slower than the float32 instruction) but read as the float32 "units" that the dense products' epilogues
// already write for the tile product (tiles.hip), and split into planes on the way into LDS.  The vertices are cut
// over blockIdx.y, every cut writes its partial matrix, and the partial matrices are added in ascending order.
// Both operands are stored "packed": in the order the instruction's lanes read them, in chunks of 32 operand rows x
// 32 of the shared index, ordered [row tile][k-block].  Lane l of a 16-deep step holds row l % 32 and k-octet
// l / 32.  A wave therefore loads a fragment as 64 consecutive 16-byte pieces, and walks through memory in one
// stream per row tile (with plain row-major operands every lane reads 32 bytes of a different row, and thousands
// of such narrow streams run side by side).  Rows and shared indices past the end are zero.
//   right operand (small, or made per call): the three planes, 6144-byte chunks [plane][step][lane][8 bfloat16]
//   left operand (the large one, streamed once from memory per product, which is what the run time follows):
//     float32, 4096-byte chunks [step][half][lane][4 floats] (half 0 = the first four of the lane's eight), split
//     into planes in registers just before use: 4 bytes per element through memory instead of 6
// X (or P = A_hat X) is constant, so its packed form is made once; W^T is packed per call.
#include "bf16_split.hpp"
#include "common.hpp"
#include "dtypes.hpp"
#include "epilogue.hpp"
#include "plane_sink.hpp"

namespace gcn {

namespace {

constexpr int BK = 32;       // shared indices per chunk
constexpr int kPlanes = 3;   // (the six products below are written out for three)
constexpr int kChunkBytes = kPlanes * (BK / 16) * 64 * 16;   // 6144: a chunk of the right operand
constexpr int kChunkVecs = kChunkBytes / 16;                 // 384
constexpr int kLeftChunkBytes = (BK / 16) * 2 * 64 * 16;     // 4096: a chunk of the left operand

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // 16 bytes in flight (a plain vector: stays in registers)

struct SplitArgs {
    const char *a;      // packed float32, a_tiles x nkb chunks
    int64_t a_tiles;
    const char *b;      // packed planes, b_tiles x nkb chunks; or (UNITS) float32 units in the tile product's order
    int b_tiles;
    int b_ld;           // UNITS: units per (32-row block, octet, half), a multiple of 32
    int64_t kb_per_split;   // 0: a workgroup runs over all of K and finishes its outputs; else blockIdx.y takes this
                            // many k-blocks and writes its own partial matrix (M x ldc, one after the other at c)
    int64_t nkb;        // k-blocks (chunks per row tile)
    float *c;
    int ldc;
    int64_t M;
    int N;
    const float *rowscale;
    Activation act;
    PlaneSink sink;         // one pass over K only: the output once more, as the tile product's operand planes
};

// One workgroup = 4 waves = 128 output rows x 32 TN columns; wave w owns rows 32 w .. 32 w + 31 of all TN column
// tiles.  Two workgroups' waves share a SIMD (<= 256 registers each), so that one wave's waits (for memory, the
// barrier, its epilogue) are another's matrix instructions:
//   - the left operand never passes through LDS: a wave loads its own fragments straight from memory, two k-blocks
//     ahead of their use, and splits them into planes in registers;
//   - the right operand (the same for all waves) goes memory -> registers, two k-blocks ahead, -> LDS, one
//     k-block ahead into the other of two LDS buffers: one barrier per k-block.  LDS holds it in packed order too,
//     so fragment reads are 64 consecutive 16-byte pieces;
//   - no load carries a condition (a guarded load makes the compiler wait for everything in flight): tiles past the
//     end read the last tile and are dropped by the epilogue, a k-block past the end re-reads the last one and is
//     never used.
constexpr int kThreads = 256;
constexpr int BM = 128;

template <int TN, bool UNITS>
__global__ __launch_bounds__(kThreads, 2) void k_gemm_split(SplitArgs g) {
    __shared__ __attribute__((aligned(16))) char Bs[2][TN * kChunkBytes];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, l32 = lane & 31;

    const int ntiles = (g.b_tiles + TN - 1) / TN;
    const int64_t mt0 = (int64_t)(blockIdx.x / ntiles) * (BM / 32) + wave;   // this wave's row tile
    const int nt0 = (blockIdx.x % ntiles) * TN;
    int64_t kb_beg = 0, kb_end = g.nkb;
    if (g.kb_per_split > 0) {
        kb_beg = (int64_t)blockIdx.y * g.kb_per_split;
        kb_end = kb_beg + g.kb_per_split < g.nkb ? kb_beg + g.kb_per_split : g.nkb;
    }

    f32x16 acc[TN];
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;

    struct AFrags {
        u32x4 f[BK / 16][2];   // eight float32 encodings per step
    };
    // Right operand per k-block.  Packed planes: TN chunks = TN x 384 vectors of 16 bytes, copied as they are.
    // UNITS (the matrix is given in the tile product's order: per block of 32 shared indices, octet kg, half and
    // column one 16-byte piece of four float32): TN x 4 x 32 (column, octet) pairs, two pieces each, split into the
    // three planes on the way into LDS, where the pair lands at lane (kg & 1) * 32 + column of step kg >> 1.
    constexpr int B_VECS = UNITS ? TN * 4 * 32 * 2 : TN * kChunkVecs;
    constexpr int B_PER = (B_VECS + kThreads - 1) / kThreads;
    static_assert(!UNITS || (B_VECS % (2 * kThreads) == 0), "whole pairs per thread");
    struct BRegs {
        u32x4 v[B_PER];
    };

    // addresses = a base that is the same for the whole wave (scalar registers) + a 32-bit byte offset per lane
    const int64_t a_tile = mt0 < g.a_tiles ? mt0 : g.a_tiles - 1;
    const char *abase = g.a + a_tile * g.nkb * kLeftChunkBytes;
    const uint32_t oa = (uint32_t)lane * 16u;
    const char *bbase = UNITS ? g.b : g.b + (int64_t)nt0 * g.nkb * kChunkBytes;
    uint32_t ob[B_PER];
    int sb[B_PER];   // UNITS: where a pair's plane 0 goes in the LDS buffer
#pragma unroll
    for (int i = 0; i < B_PER; ++i) {
        if (UNITS) {
            const int pair = tid + (i / 2) * kThreads, half = i & 1;
            const int c32 = pair % 32, kg = (pair / 32) % 4, t = pair / 128;
            const int col = (nt0 + t < g.b_tiles ? nt0 + t : g.b_tiles - 1) * 32 + c32;
            ob[i] = (uint32_t)(((kg * 2 + half) * g.b_ld + col) * 16);
            sb[i] = t * kChunkBytes + ((kg >> 1) * 64 + (kg & 1) * 32 + c32) * 16;
        } else {
            const int v = (tid + i * kThreads) % B_VECS;   // threads past the end load again what others load
            const int t = v / kChunkVecs, w = v % kChunkVecs;
            const int tile = nt0 + t < g.b_tiles ? t : g.b_tiles - 1 - nt0;
            ob[i] = (uint32_t)((int64_t)tile * g.nkb * kChunkBytes + w * 16);
            sb[i] = 0;
        }
    }
    const int64_t kb_last = kb_end - 1;
    const int64_t b_block = UNITS ? (int64_t)8 * g.b_ld * 16 : kChunkBytes;   // bytes of the right operand per k-block

    auto load_a = [&](AFrags &fr, int64_t kb) {
        kb = kb < kb_last ? kb : kb_last;
        const char *base = abase + kb * kLeftChunkBytes;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks)
#pragma unroll
            for (int q = 0; q < 2; ++q)
                fr.f[ks][q] = *reinterpret_cast<const u32x4 *>(base + oa + (ks * 2 + q) * 1024);
    };
    auto load_b = [&](BRegs &rb, int64_t kb) {
        kb = kb < kb_last ? kb : kb_last;
        const char *base = bbase + kb * b_block;
#pragma unroll
        for (int i = 0; i < B_PER; ++i) rb.v[i] = *reinterpret_cast<const u32x4 *>(base + ob[i]);
    };
    auto stash_b = [&](const BRegs &rb, const int buf) {
        if (UNITS) {
#pragma unroll
            for (int i = 0; i + 1 < B_PER; i += 2) {
                const uint32_t x[8] = {rb.v[i][0],     rb.v[i][1],     rb.v[i][2],     rb.v[i][3],
                                       rb.v[i + 1][0], rb.v[i + 1][1], rb.v[i + 1][2], rb.v[i + 1][3]};
                uint4 o[kPlanes];
                split_column<kPlanes>(x, o);
#pragma unroll
                for (int p = 0; p < kPlanes; ++p)
                    *reinterpret_cast<uint4 *>(&Bs[buf][sb[i] + p * (BK / 16) * 1024]) = o[p];
            }
        } else {
#pragma unroll
            for (int i = 0; i < B_PER; ++i)
                if (B_VECS % kThreads == 0 || tid + i * kThreads < B_VECS)
                    *reinterpret_cast<u32x4 *>(&Bs[buf][(tid + i * kThreads) * 16]) = rb.v[i];
        }
    };
    auto right = [&](const int buf, const int t, const int ks, const int p) {
        return *reinterpret_cast<const bf16x8 *>(&Bs[buf][t * kChunkBytes + (p * (BK / 16) + ks) * 1024 + lane * 16]);
    };
    auto compute = [&](const AFrags &fr, const int buf) {
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 af[kPlanes];
            {
                const uint32_t x[8] = {fr.f[ks][0][0], fr.f[ks][0][1], fr.f[ks][0][2], fr.f[ks][0][3],
                                       fr.f[ks][1][0], fr.f[ks][1][1], fr.f[ks][1][2], fr.f[ks][1][3]};
                uint4 o[kPlanes];
                split_column<kPlanes>(x, o);
#pragma unroll
                for (int p = 0; p < kPlanes; ++p) {
                    union {
                        uint4 u;
                        bf16x8 v;
                    } cv;
                    cv.u = o[p];
                    af[p] = cv.v;
                }
            }
            // smallest terms first; two column tiles alternate, so that no instruction waits for the one before it
            if (TN >= 2) {
#pragma unroll
                for (int t = 0; t + 1 < TN; t += 2) {
                    bf16x8 b0[kPlanes], b1[kPlanes];
#pragma unroll
                    for (int p = 0; p < kPlanes; ++p) {
                        b0[p] = right(buf, t, ks, p);
                        b1[p] = right(buf, t + 1, ks, p);
                    }
#define GCN_TERM(I, J)                                                                           \
    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[I], b0[J], acc[t], 0, 0, 0);             \
    acc[t + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[I], b1[J], acc[t + 1], 0, 0, 0);
                    GCN_TERM(2, 0)
                    GCN_TERM(1, 1)
                    GCN_TERM(0, 2)
                    GCN_TERM(1, 0)
                    GCN_TERM(0, 1)
                    GCN_TERM(0, 0)
#undef GCN_TERM
                }
            } else {
                bf16x8 b0[kPlanes];
#pragma unroll
                for (int p = 0; p < kPlanes; ++p) b0[p] = right(buf, 0, ks, p);
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[2], b0[0], acc[0], 0, 0, 0);
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[1], b0[1], acc[0], 0, 0, 0);
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[0], b0[2], acc[0], 0, 0, 0);
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[1], b0[0], acc[0], 0, 0, 0);
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[0], b0[1], acc[0], 0, 0, 0);
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[0], b0[0], acc[0], 0, 0, 0);
            }
        }
    };
    static_assert(kPlanes == 3 && (TN == 1 || TN % 2 == 0), "the products above are written out for three planes");

    if (kb_beg < kb_end) {   // (a split past the end of K has nothing to add and writes zeros)
        // Loads run two k-blocks ahead of their use: three register sets for each operand, taken in turn.  (A set
        // is never copied: a copy would have to wait for the loads into it.)
        AFrags f0, f1, f2;
        BRegs b0, b1, b2;
        int buf = 0;
        // k-block kb: `use` holds its left fragments and LDS buffer `buf` its right operand; `put` holds the right
        // operand of kb + 1, loaded a step ago, and goes to the other buffer; `fill` and `get` take kb + 2
        auto step = [&](const AFrags &use, AFrags &fill, const BRegs &put, BRegs &get, int64_t kb) {
            load_a(fill, kb + 2);
            load_b(get, kb + 2);
            __builtin_amdgcn_sched_barrier(0);   // the loads go out before the products, not after them
            compute(use, buf);
            stash_b(put, buf ^ 1);
            __syncthreads();   // the other buffer is complete, and everyone is done reading this one
            buf ^= 1;
        };
        load_a(f0, kb_beg);
        load_b(b0, kb_beg);
        load_a(f1, kb_beg + 1);
        load_b(b1, kb_beg + 1);
        stash_b(b0, 0);
        __syncthreads();
        int64_t kb = kb_beg;
#pragma unroll 1
        for (; kb + 3 <= kb_end; kb += 3) {
            step(f0, f2, b1, b2, kb);
            step(f1, f0, b2, b0, kb + 1);
            step(f2, f1, b0, b1, kb + 2);
        }
        if (kb < kb_end) step(f0, f2, b1, b2, kb);
        if (kb + 1 < kb_end) step(f1, f0, b2, b0, kb + 1);
    }

    float *cbase = g.c;
    if (g.kb_per_split > 0) cbase += (int64_t)blockIdx.y * g.M * g.ldc;   // this split's partial matrix
    const bool to_sink = g.sink.planes != nullptr && g.kb_per_split == 0;
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        const int col = (nt0 + t) * 32 + l32;
        float xs[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int64_t row = mt0 * 32 + 8 * (v / 4) + 4 * h + (v % 4);
            float x = 0.0f;
            if (row < g.M && col < g.ldc) {
                x = col < g.N ? acc[t][v] : 0.0f;
                if (g.kb_per_split == 0) {
                    if (g.rowscale) x *= g.rowscale[row];
                    x = activate(x, g.act, row, col);
                }
                cbase[row * g.ldc + col] = x;
            }
            xs[v] = x;
        }
        if (to_sink) sink_store(g.sink, mt0 * 32, col, h, xs);
    }
}

// where the eight values (operand row `row`, shared indices 8 oct .. 8 oct + 7) go in a packed operand of nkb
// k-blocks: right operand: plane 0, the other planes follow 2048 bytes apart; left operand: the first four floats,
// the other four follow 1024 bytes apart
template <bool LEFT>
__device__ inline size_t packed_offset(int64_t row, int64_t oct, int64_t nkb) {
    const int64_t tile = row >> 5, kb = oct >> 2;
    const int ks = (int)(oct >> 1) & 1, hh = (int)oct & 1;
    const int lane = hh * 32 + (int)(row & 31);
    if (LEFT) return (size_t)(tile * nkb + kb) * kLeftChunkBytes + (size_t)((ks * 128 + lane) * 16);
    return (size_t)(tile * nkb + kb) * kChunkBytes + (size_t)((ks * 64 + lane) * 16);
}

template <bool LEFT>
__device__ inline void store_packed(char *dst, int64_t row, int64_t oct, int64_t nkb, const uint32_t (&x)[8]) {
    char *at = dst + packed_offset<LEFT>(row, oct, nkb);
    if (LEFT) {
        *reinterpret_cast<uint4 *>(at) = make_uint4(x[0], x[1], x[2], x[3]);
        *reinterpret_cast<uint4 *>(at + 1024) = make_uint4(x[4], x[5], x[6], x[7]);
    } else {
        uint4 o[kPlanes];
        split_column<kPlanes>(x, o);
#pragma unroll
        for (int p = 0; p < kPlanes; ++p) *reinterpret_cast<uint4 *>(at + p * 2048) = o[p];
    }
}

// packed operand whose rows are the rows of src [rows x cols]: one thread per row and octet of columns; operand
// rows up to a whole tile and shared indices up to a whole k-block are written as zero
template <bool LEFT>
__global__ __launch_bounds__(256) void k_pack_rows(const float *__restrict__ src, int ld, int64_t rows, int cols,
                                                   char *__restrict__ dst, int64_t tiles, int64_t nkb) {
    const int64_t octs = nkb * 4;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= tiles * 32 * octs) return;
    const int64_t r = i / octs, oct = i % octs;
    uint32_t x[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
        x[j] = (r < rows && oct * 8 + j < cols) ? __float_as_uint(src[r * ld + oct * 8 + j]) : 0u;
    store_packed<LEFT>(dst, r, oct, nkb, x);
}

// packed operand whose rows are the columns of src [rows x cols] (the shared index runs over src's rows): a
// workgroup takes 64 rows x 32 columns of src through LDS; thread (column c, octet of rows) then writes its
// pieces, the 32 columns of a tile side by side
template <bool LEFT>
__global__ __launch_bounds__(256) void k_pack_transposed(const float *__restrict__ src, int ld, int64_t rows,
                                                         int cols, char *__restrict__ dst, int64_t nkb) {
    __shared__ float tile[64][33];
    const int64_t r0 = (int64_t)blockIdx.x * 64;
    const int c0 = blockIdx.y * 32;
    for (int i = threadIdx.x; i < 64 * 32; i += 256) {
        const int r = i / 32, c = i % 32;
        tile[r][c] = (r0 + r < rows && c0 + c < cols) ? src[(r0 + r) * ld + c0 + c] : 0.0f;
    }
    __syncthreads();
    const int c = threadIdx.x % 32, kg = threadIdx.x / 32;
    if (r0 + kg * 8 >= nkb * BK) return;   // (the last workgroup may reach past the last k-block)
    uint32_t x[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) x[j] = __float_as_uint(tile[kg * 8 + j][c]);
    store_packed<LEFT>(dst, c0 + c, r0 / 8 + kg, nkb, x);
}

}  // namespace

size_t packed_bytes(int64_t rows, int64_t k, bool left) {
    return (size_t)((rows + 31) / 32) * (size_t)((k + BK - 1) / BK) * (left ? kLeftChunkBytes : kChunkBytes);
}

int pack_rows(const float *src, int ld, int64_t rows, int cols, void *dst, bool left, hipStream_t st) {
    if (rows <= 0 || cols <= 0) return GCN_OK;
    const int64_t tiles = (rows + 31) / 32, nkb = (cols + BK - 1) / BK;
    const int64_t items = tiles * 32 * nkb * 4;
    const dim3 grid((unsigned)((items + 255) / 256));
    if (left) k_pack_rows<true><<<grid, dim3(256), 0, st>>>(src, ld, rows, cols, (char *)dst, tiles, nkb);
    else k_pack_rows<false><<<grid, dim3(256), 0, st>>>(src, ld, rows, cols, (char *)dst, tiles, nkb);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int pack_transposed(const float *src, int ld, int64_t rows, int cols, void *dst, bool left, hipStream_t st) {
    if (rows <= 0 || cols <= 0) return GCN_OK;
    const int64_t nkb = (rows + BK - 1) / BK;
    // whole tiles of 32 operand rows: the columns past `cols` of the last tile are written as zero
    const dim3 grid((unsigned)((nkb * BK + 63) / 64), (unsigned)((cols + 31) / 32));
    if (left) k_pack_transposed<true><<<grid, dim3(256), 0, st>>>(src, ld, rows, cols, (char *)dst, nkb);
    else k_pack_transposed<false><<<grid, dim3(256), 0, st>>>(src, ld, rows, cols, (char *)dst, nkb);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

namespace {
int tn_split_count(int64_t M, int64_t K, int N) {
    const int bn = N > 64 ? 128 : 64;
    const int64_t tiles = (M + BM - 1) / BM * ((N + bn - 1) / bn);
    int64_t splits = tunable("split_tn_wgs", 256) / (tiles > 0 ? tiles : 1);   // one workgroup per compute unit (measured better than two: fewer partial matrices)
    const int64_t max_by_k = (K + 8 * BK - 1) / (8 * BK);   // at least 256 of the shared index per split
    if (splits > max_by_k) splits = max_by_k;
    return splits < 1 ? 1 : (int)splits;
}
}  // namespace

int gemm_split(const void *a, const void *b, float *c, int ldc, int64_t M, int64_t K, int N, const float *rowscale,
               const Activation *act, hipStream_t st, const PlaneSink *sink) {
    if (M <= 0) return GCN_OK;
    if (K <= 0 || N <= 0 || ldc % 16 != 0 || N > ldc) {
        set_error("gemm_split: bad shape M=%lld K=%lld N=%d ldc=%d", (long long)M, (long long)K, N, ldc);
        return GCN_EINVAL;
    }
    const int64_t nkb = (K + BK - 1) / BK;
    SplitArgs g{(const char *)a, (M + 31) / 32, (const char *)b, (N + 31) / 32, 0, 0, nkb, c, ldc, M, N, rowscale,
                act ? *act : Activation{kActNone, 0, 0u, 1.0f, 0ull}, sink ? *sink : PlaneSink{nullptr, 0, 0}};
    const unsigned mtiles = (unsigned)((M + BM - 1) / BM);
    if (N > 64)
        k_gemm_split<4, false><<<dim3(mtiles * (unsigned)((N + 127) / 128)), dim3(kThreads), 0, st>>>(g);
    else if (N > 32)
        k_gemm_split<2, false><<<dim3(mtiles), dim3(kThreads), 0, st>>>(g);
    else
        k_gemm_split<1, false><<<dim3(mtiles), dim3(kThreads), 0, st>>>(g);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

size_t gemm_split_tn_partial_floats(int64_t M, int64_t K, int N) {
    return (size_t)tn_split_count(M, K, N) * (size_t)M * (size_t)padded_width(N);
}

int gemm_split_tn(const void *a, const void *b_units, int b_ld, float *c, int ldc, int64_t M, int64_t K, int N,
                  float *partials, size_t partial_floats, hipStream_t st) {
    if (M <= 0) return GCN_OK;
    if (K <= 0 || N <= 0 || ldc % 16 != 0 || N > ldc || b_ld % 32 != 0 || b_ld < N) {
        set_error("gemm_split_tn: bad shape M=%lld K=%lld N=%d ldc=%d units ld=%d", (long long)M, (long long)K, N, ldc,
                  b_ld);
        return GCN_EINVAL;
    }
    const int64_t nkb = (K + BK - 1) / BK;
    const int splits = tn_split_count(M, K, N);
    if (!partials || (size_t)splits * (size_t)M * (size_t)ldc > partial_floats) {
        set_error("gemm_split_tn: partial buffer too small");
        return GCN_EWORKSPACE;
    }
    SplitArgs g{(const char *)a, (M + 31) / 32, (const char *)b_units, b_ld / 32, b_ld, (nkb + splits - 1) / splits, nkb,
                partials, ldc, M, N, nullptr, Activation{kActNone, 0, 0u, 1.0f, 0ull}, PlaneSink{nullptr, 0, 0}};
    const unsigned mtiles = (unsigned)((M + BM - 1) / BM);
    const unsigned ys = (unsigned)splits;
    if (N > 64)
        k_gemm_split<4, true><<<dim3(mtiles * (unsigned)((N + 127) / 128), ys), dim3(kThreads), 0, st>>>(g);
    else   // (one column tile would leave half the threads without a pair to load: it runs as two, the second clamped)
        k_gemm_split<2, true><<<dim3(mtiles, ys), dim3(kThreads), 0, st>>>(g);
    GCN_LAUNCH_CHECK();
    return reduce_partials(partials, splits, (size_t)M * (size_t)ldc, c, st);
}

}  // namespace gcn

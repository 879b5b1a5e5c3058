// Internal declarations shared by the translation units of libgcn355.so (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "../../include/gcn355.h"
#include "../../include/gcn355_debug.h"
#include "epilogue.hpp"

namespace gcn {

void set_error(const char *fmt, ...);

// Named integer knobs for benchmark sweeps (gcn_set_tunable); unknown names read as the default.
int64_t tunable(const char *name, int64_t fallback);

#define GCN_HIP(call)                                                                          \
    do {                                                                                       \
        hipError_t e_ = (call);                                                                \
        if (e_ != hipSuccess) {                                                                \
            gcn::set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
            return GCN_EHIP;                                                                   \
        }                                                                                      \
    } while (0)

#define GCN_LAUNCH_CHECK()                                                                     \
    do {                                                                                       \
        hipError_t e_ = hipGetLastError();                                                     \
        if (e_ != hipSuccess) {                                                                \
            gcn::set_error("kernel launch failed: %s (%s:%d)", hipGetErrorString(e_), __FILE__, __LINE__); \
            return GCN_EHIP;                                                                   \
        }                                                                                      \
    } while (0)

constexpr int kWave = 64;
constexpr int kLdAlign = 16;   // leading dimensions are multiples of 16 elements (64 B in fp32)
constexpr int kColSlack = 64;  // readable entries after the last column index (index prefetch runs one step ahead)
constexpr int kHeavyDegree = 32;  // rows with at least this many entries get a whole wave in the aggregation
constexpr int kSplitDegree = 4096; // rows with more entries than this are cut into chunks, one wave per chunk
constexpr int kChunk = 2048;       // entries per chunk of a split row
constexpr int kXcds = 8;       // workgroup ids are dealt round-robin to 8 XCDs, each with its own L2
constexpr int kRangesPerXcd = 2;  // column ranges of the phased aggregation schedule per XCD
constexpr int kColBlocks = kXcds * kRangesPerXcd;
constexpr int kTileRows = 128;             // a dense tile covers this many rows by 32 columns
constexpr int kTileMinEntriesFloor = 64;   // a dense tile holds at least this many entries (bounds their number)
constexpr int kTileMinEntriesDefault = 64; // the break-even of one tile product against gathering its entries
constexpr int kTileRunMin = 16;            // a row block with up to 1.5 x this many tiles is never cut into runs
constexpr int kTileChunkMin = 8;           // runs are no shorter than this

inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }
inline int padded_width(int w) { return (int)round_up(w, kLdAlign); }

// Bump allocator over a caller workspace; with base == nullptr it only measures.
struct Carver {
    char *base;
    size_t off = 0;
    explicit Carver(void *b) : base((char *)b) {}
    template <typename T>
    T *take(size_t count) {
        off = (off + 255) & ~(size_t)255;
        T *p = base ? (T *)(base + off) : nullptr;
        off += count * sizeof(T);
        return p;
    }
    size_t bytes() const { return (off + 255) & ~(size_t)255; }
};

// ---------------------------------------------------------------------------------------------
// Graph preparation (prep.hip)
struct PrepBuffers {
    // canonical pattern of A + I
    int64_t *rowptr;   // n + 1
    int32_t *col;      // <= nnz_in + n
    int32_t *deg;      // n
    float *dinv;       // n
    // schedule: heavy rows (kHeavyDegree <= degree <= kSplitDegree) first, then light rows, then split rows (degree >
    // kSplitDegree), each class in ascending vertex order
    int32_t *perm;     // n   slot -> row
    // split rows: row number j of that class (perm[n_heavy + n_light + j]) owns the chunks chunk_off[j] .. chunk_off[j + 1],
    // chunk k of it covering entries [k kChunk, (k + 1) kChunk) of the row; chunk_srow[c] = j
    int64_t split_cap = 0, chunk_cap = 0;   // capacities (from the number of stored entries)
    int32_t *split_cnt;   // split_cap
    int64_t *chunk_off;   // split_cap + 1
    int32_t *chunk_srow;  // chunk_cap
    int64_t *lpos;     // n + 1   exclusive prefix of the light flags (scratch)
    // heavy rows are handed to the XCDs in contiguous runs of about equal numbers of entries (not rows): XCD x takes
    // the schedule slots xcd_start[x] .. xcd_start[x + 1]
    int32_t *xcd_start;   // kXcds + 1
    int32_t *row_start;   // kXcds + 1: contiguous id ranges with equal numbers of entries (phased schedule)
    // column blocks: the ids are cut into kColBlocks equal ranges; segoff[r * (kColBlocks + 1) + b] is the offset,
    // from the start of row r, of its first column in range b (and the row length for b = kColBlocks)
    int32_t *segoff;   // n * (kColBlocks + 1); null for graphs too large for the phased schedule
    // phased schedule (only for graphs small enough for it, else unused): rows of each wave, see phased_shape()
    int32_t *prow;     // kXcds * W * R
    // scratch
    int32_t *scratch;  // nnz_in + n
    int32_t *heavy;    // n   1 if the row is heavy
    int64_t *hpos;     // n + 1   exclusive prefix of heavy[]
    int64_t *blocksum; // scan partials
    int32_t *flags;    // 16 ints: [0] graph error, [1] label error, [2] n_train, [3] max degree, [4] heavy rows, [5] light rows
};

int prep_validate(int64_t n, int64_t nnz_in, const int64_t *rowptr, const int32_t *col, int32_t *flags,
                  hipStream_t st);
int prep_canonical(int64_t n, int64_t nnz_in, const int64_t *rowptr, const int32_t *col, PrepBuffers &pb,
                   hipStream_t st);
int prep_schedule(int64_t n, PrepBuffers &pb, hipStream_t st);
// dst's pattern (rowptr, col, deg) = src's entries whose column c has keep[c] != 0, rows in the same order
int prep_keep_columns(int64_t n, const PrepBuffers &src, const uint8_t *keep, PrepBuffers &dst, hipStream_t st);
// Phased aggregation schedule: XCD x owns the rows row_start[x] .. row_start[x + 1] (contiguous id ranges holding
// equal numbers of entries), each of its W waves R of them.  Not available when an XCD would own more than
// kPhasedMaxRows rows: 8 rows per wave with 896 waves per XCD (32 CUs x 4 SIMDs x 7 waves, what the kernel's
// register use lets be resident at once; the schedule likes the whole grid resident).
constexpr int kPhasedMaxRows = 8 * 896;
inline bool phased_possible(int64_t n) { return n <= (int64_t)kXcds * kPhasedMaxRows; }   // decides the allocation
inline bool phased_shape(int64_t max_rows_per_xcd, int *W, int *R) {
    const int64_t need = (max_rows_per_xcd + 895) / 896;
    if (max_rows_per_xcd < 1 || need > 8) return false;
    *R = need <= 4 ? 4 : (need <= 6 ? 6 : 8);
    *W = (int)((max_rows_per_xcd + *R - 1) / *R);
    return true;
}
int prep_balance_rows(int64_t n, const int32_t *deg, const int32_t *row_start, int W, int R, int32_t *prow,
                      hipStream_t st);
// ---------------------------------------------------------------------------------------------
// Dense tiles (kTileRows x 32) of the adjacency pattern (tiles.hip)
struct TileBuffers {
    int64_t n_rb = 0;       // row blocks = ceil(n / kTileRows)
    int64_t capacity = 0;   // dense tiles the arrays can hold
    int32_t *tile_cnt = nullptr;   // n_rb: dense tiles of each row block
    int64_t *tile_ptr = nullptr;   // n_rb + 1: exclusive prefix of tile_cnt
    int32_t *tile_col = nullptr;   // capacity: column tile (32 columns) of each dense tile, ascending inside a row block
    int32_t *tile_rt = nullptr;    // capacity: row block of each dense tile
    uint32_t *bits = nullptr;      // capacity * kTileRows: word r of tile k = columns that row r of the tile holds
    unsigned long long *totals = nullptr;   // [0] stored entries inside the dense tiles
    // the product's work items (runs of tiles of one row block) and the row blocks whose runs must be added up
    size_t item_capacity = 0;
    void *items = nullptr;         // item_capacity x 4 int32
    void *folds = nullptr;         // n_rb x 4 int32
    int32_t n_items = 0, n_folds = 0, n_slots = 0;   // n_slots: blocks of kTileRows rows in the partial-sum buffer
};
size_t tiles_capacity(int64_t entries);
size_t tiles_item_capacity(int64_t n_rb, int64_t tile_capacity);
// fills tile_cnt, tile_ptr, tile_col, tile_rt and totals from the canonical pattern
int tiles_select(int64_t n, const int64_t *rowptr, const int32_t *col, int min_entries, TileBuffers &tb,
                 int64_t *blocksum, hipStream_t st);
// fills bits, and res.deg / res.rowptr / res.col with the entries outside the dense tiles
int tiles_build(int64_t n, const int64_t *rowptr, const int32_t *col, int64_t n_tiles, TileBuffers &tb,
                PrepBuffers &res, hipStream_t st);
// fills items / folds and their counts from a host copy of tile_ptr (synchronous)
int tiles_plan(const std::vector<int64_t> &tile_ptr, TileBuffers &tb, hipStream_t st);

int prep_labels_mask(int64_t n, const int32_t *labels, const uint8_t *mask, int32_t n_classes, int32_t *labels_out,
                     uint8_t *mask_out, int32_t *flags, hipStream_t st);
size_t scan_blocks(int64_t n);
// out[i] = in[0] + ... + in[i-1] for i = 0..n (n + 1 outputs); blocksum holds scan_blocks(n) words
int exclusive_scan_i32(int64_t n, const int32_t *in, int64_t *out, int64_t *blocksum, hipStream_t st);

// ---------------------------------------------------------------------------------------------
// Subgraph approximation (augment.hip)
size_t augment_workspace_bytes(int64_t n);
int augment_partition(int64_t n, const int64_t *rowptr, const int32_t *col, const int32_t *part, int32_t n_parts,
                      int32_t p, double overlap, uint64_t seed, void *workspace, int64_t *n_out, int64_t *n_local_out,
                      int64_t *nnz_out, int32_t *vertices, int64_t *rowptr_out, int32_t *col_out, hipStream_t st);
int gather_rows(const void *src, size_t row_bytes, const int32_t *idx, int64_t n_idx, void *dst, hipStream_t st);

// ---------------------------------------------------------------------------------------------
// Layout helpers (elementwise.hip).  "padded" = row-major with leading dimension ld >= width, pad zero.
// dst / src element type is float (GCN_F32) or bfloat16 (GCN_BF16); the caller-side matrix is always float.
int pad_rows(const float *src, int64_t rows, int width, void *dst, int dst_dtype, int ld, const float *rowscale,
             hipStream_t st);
int unpad_rows(const void *src, int src_dtype, int ld, int64_t rows, int width, float *dst, const float *rowdiv,
               hipStream_t st);
// bfloat16 copies of w [rows x ld]: same layout (wb) and transposed [ld x ld_t] (wbt)
int weight_copies(const float *w, int rows, int ld, void *wb, void *wbt, int ld_t, hipStream_t st);
int fill_zero(void *p, size_t bytes, hipStream_t st);
// dst[r, :] = rowscale[r] * src[r, :] for matrices of the same storage type and leading dimension
int scale_rows(const void *src, void *dst, int dtype, int64_t rows, int ld, const float *rowscale, hipStream_t st);

// Loss / accuracy / dLoss/dlogits (scaled by dinv for the aggregation that follows).
constexpr int kLossBlocks = 4096;
int loss_forward(int64_t n, int classes, const float *logits, int ld, const int32_t *labels, const uint8_t *mask,
                 const float *dinv, int64_t n_train, void *dzs, int dz_dtype, int ld_dz, double *loss_part,
                 long long *corr_part, float *result /* [0] loss, [1] accuracy, as float */,
                 long long *result_correct, hipStream_t st, const struct PlaneSink *sink = nullptr);
// whether loss_forward writes dLoss/dlogits through a sink for this shape (at most 64 classes, float32)
bool loss_can_sink(int classes, int dz_dtype);
// w_l -= lr dw_l for every layer l in one launch; end[l] = number of elements of layers 0..l together
constexpr int kMaxLayers = 16;
struct SgdLayers {
    float *w[kMaxLayers];
    const float *dw[kMaxLayers];
    size_t end[kMaxLayers];
    int n;
};
int sgd_update(const SgdLayers &ls, float lr, hipStream_t st);
int adam_update(float *w, const float *dw, float *m, float *v, size_t count, float lr, float beta1, float beta2,
                float eps, int64_t step, hipStream_t st);
// every weights[i][0..elems) becomes the mean over i (summed in list order)
int average_in_place(float *const *weights, int count, size_t elems, hipStream_t st);
int calibration_copy(const void *src, void *dst, size_t bytes, hipStream_t st);
int xcc_ids(int32_t *out, int n_blocks, hipStream_t st);

// ---------------------------------------------------------------------------------------------
// Aggregation (spmm.hip):  out[r, :] = dinv[r] * sum over the columns c of row r of  t[c, :],
// where t already carries the factor dinv[c] and has an all-zero row n that stands in for entries
// past the end of a row.  Rows are taken in schedule order: perm[0 .. n_heavy) one wave each, the rest
// one lane group each.
enum SpmmEpilogue { kEpiNone = 0, kEpiRelu = 1 };
struct SpmmArgs {
    const int64_t *rowptr;
    const int32_t *col;     // kColSlack readable entries follow the last one
    const int32_t *perm;
    const float *dinv;
    const int32_t *segoff;  // column-block offsets per row (see PrepBuffers)
    const int32_t *prow;    // rows per wave of the phased schedule, or null
    int phased_w, phased_r; // waves per XCD and rows per wave of that schedule (0: not available)
    int64_t n;
    int64_t n_heavy;    // rows with a wave each
    int64_t n_light;    // rows with a lane group each
    int64_t n_split;    // rows cut into chunks (n_heavy + n_light + n_split = n)
    int64_t n_chunks;
    const int32_t *xcd_start;   // kXcds + 1 slots: the heavy rows of each XCD
    int64_t xcd_rows_max;       // the longest of those runs
    const int64_t *chunk_off;
    const int32_t *chunk_srow;
    float *chunk_sums;  // n_chunks x cols floats: the chunks' sums (workspace of the call)
    const void *t;      // float or bfloat16, ld_t elements per row, n + 1 rows
    int t_dtype;
    int ld_t;
    void *out;          // float or bfloat16 (bfloat16 only from a bfloat16 input)
    int out_dtype;
    int ld_out;
    int cols;           // columns handled by this launch (multiple of 8, <= both leading dimensions)
    int width;          // true width of the whole matrix (element numbering of the dropout mask)
    int epilogue;
    // dropout (epilogue kEpiRelu, training): threshold 0 = keep everything
    uint32_t drop_threshold;
    float keep_scale;
    uint64_t drop_key;
    // Dense tiles (tile_ptr null: none).  With tiles, rowptr / col / perm / segoff / prow describe the residual
    // pattern, and the launch first writes the tiles' sums to out, then adds the residual rows and finishes.
    const int64_t *tile_ptr;
    const int32_t *tile_col;
    const uint32_t *bits;
    const void *tile_items;   // work items of the tile product and their number
    int32_t n_items;
    const void *tile_folds;   // row blocks whose runs are added up afterwards
    int32_t n_folds, n_slots;
    float *tile_partial;      // n_slots x kTileRows x cols floats
    void *tile_planes;        // tiles_plane_bytes(n, cols, t_dtype): the input in the order the tile product reads it
    // Overlap of the two parts (all four set, or none): the tile product runs on `side` into tile_sums [n x cols
    // floats] while the gather kernel writes plain sums to out on the caller's stream; a third launch adds the two
    // and finishes the rows.  Without them the gather kernel follows the tile product and finishes the rows itself.
    float *tile_sums;
    float *gather_sums;   // [n x cols floats] the gather kernel's plain sums when the output itself is bfloat16
    hipStream_t side;
    hipEvent_t ev_fork, ev_join;
    int finish_mode;     // set by spmm_launch, see SpmmFinish
    int planes_ready;    // tile_planes already holds this input (its producer wrote it through a PlaneSink)
    int spread;          // the pattern was searched for dense tiles and has next to none: no community keeps its
                         // vertices together, a row's entries are taken to be spread evenly over all columns
};
// Where the producer of an aggregation's float32 input also leaves it in the order the tile product reads it
// (planes == nullptr: nowhere); n_ct blocks of 32 rows, per block and k-octet `ld` units of two 16-byte halves.
struct PlaneSink {
    void *planes;
    int n_ct;
    int ld;
};
// the sink for aggregation `a` (knob "fused_planes", default 1), or none when that aggregation runs no tile product
// over float32 input
PlaneSink tiles_plane_sink(const SpmmArgs &a);
// what the gather kernels do with a row's sum
enum SpmmFinish {
    kFinishRow = 0,      // scale by d_i^-1/2, activation, store
    kFinishAddStored = 1,  // first add what the output already holds (the tiles' sums), then as above
    kFinishPlainSum = 2    // store the plain sum (float32 output); a later launch finishes the rows
};
size_t tiles_plane_bytes(int64_t n, int cols, int dtype);
// the aggregation's input in the order the tile product reads it, unless its producer has written that
int tiles_planes(const SpmmArgs &a, hipStream_t st);
// a float32 matrix t [n x cols] (cols even) in that order: units of tiles_plane_bytes(n, cols, GCN_F32) bytes
int units_from_rows(const float *t, int ld_t, int64_t n, int cols, void *units, hipStream_t st);
// dst [n x ld_dst] = the sums over the dense tiles only (float32, no scaling); after tiles_planes
int tiles_launch(const SpmmArgs &a, float *dst, int ld_dst, hipStream_t st);
int spmm_launch(const SpmmArgs &a, hipStream_t st);

// ---------------------------------------------------------------------------------------------
// Dense products on the matrix cores (gemm.hip).  All leading dimensions are multiples of 16 and the
// padding columns/rows of the operands are zero.
//   nn:  c[m, :] = act(rowscale[m] * (a[m, :] b))           a: M x K,  b: K x N,  c: M x N
//   nt:  c[m, :] = rowscale[m] * scale * [gate[m, :] > 0] * (a[m, :] b^T)      b: N x K
//   tn:  c = a^T b  reduced over the M rows of a and b in fixed order (split over row ranges)
// nn and nt also leave their output in *sink when one is given (plane_sink.hpp)
int gemm_nn(const float *a, int lda, const float *b, int ldb, float *c, int ldc, int64_t M, int K, int N,
            const float *rowscale, const Activation *act /* may be null */, hipStream_t st,
            const PlaneSink *sink = nullptr);
int gemm_nt(const float *a, int lda, const float *b, int ldb, float *c, int ldc, int64_t M, int K, int N,
            const float *rowscale, const float *gate, int ldg, float scale, hipStream_t st,
            const PlaneSink *sink = nullptr);
// nn for few rows: c = [relu](a b) with the shared dimension split over workgroups and the partial matrices added
// in ascending order; partials holds gemm_nn_splitk_partial_floats(M, K, N) floats
size_t gemm_nn_splitk_partial_floats(int64_t M, int K, int N);
int gemm_nn_splitk(const float *a, int lda, const float *b, int ldb, float *c, int ldc, int64_t M, int K, int N,
                   bool relu, float *partials, size_t partial_floats, hipStream_t st);
size_t gemm_tn_partial_floats(int64_t rows, int M, int N);
int gemm_tn(const float *a, int lda, const float *b, int ldb, float *c, int ldc, int64_t rows, int M, int N,
            float *partials, size_t partial_floats, hipStream_t st);

int reduce_partials(const float *partials, int splits, size_t count, float *c, hipStream_t st);

// bfloat16 operands, float32 accumulation (gemm_bf16.hip).  a, b, c, gate are bfloat16 matrices; bt / b hold the
// second operand with the shared dimension contiguous: nn takes W^T [N x K], nt takes W [N x K].
int gemm_bf16_nn(const void *a, int lda, const void *bt, int ldb, void *c, int ldc, int64_t M, int K, int N,
                 const float *rowscale, const Activation *act /* may be null */, hipStream_t st);
int gemm_bf16_nt(const void *a, int lda, const void *b, int ldb, void *c, int ldc, int64_t M, int K, int N,
                 const float *rowscale, const void *gate, int ldg, float scale, hipStream_t st);
size_t gemm_bf16_tn_partial_floats(int64_t rows, int M, int N);
int gemm_bf16_tn_partials(const void *a, int lda, const void *b, int ldb, int ldc, int64_t rows, int M, int N,
                          float *partials, size_t partial_floats, int *splits_out, hipStream_t st);

// float32 products on the bfloat16 matrix instruction (gemm_split.hip).  A "packed" operand holds a float32 matrix
// [rows x k] in the order the instruction's lanes read it, padded with zeros to whole tiles of 32 rows and 32
// shared indices: the left operand of a product as float32 (split into three bfloat16 planes in registers), the
// right operand as the three planes; packed_bytes(rows, k, left) bytes.
size_t packed_bytes(int64_t rows, int64_t k, bool left);
// the operand whose rows are src's rows (src [rows x cols], shared index = column)
int pack_rows(const float *src, int ld, int64_t rows, int cols, void *dst, bool left, hipStream_t st);
// the operand whose rows are src's columns (shared index = src's row)
int pack_transposed(const float *src, int ld, int64_t rows, int cols, void *dst, bool left, hipStream_t st);
// c [M x N] = act(rowscale * (a b^T)), a [M x K] packed left, b [N x K] packed right
int gemm_split(const void *a, const void *b, float *c, int ldc, int64_t M, int64_t K, int N, const float *rowscale,
               const Activation *act /* may be null */, hipStream_t st, const PlaneSink *sink = nullptr);
// c [M x N] = a b, a [M x K] packed left, b [K x N] as float32 units in the tile product's order (tiles.hip:
// units_from_rows; b_ld units per octet and half).  K is cut over workgroups; the partial matrices are added in
// ascending order.  partials holds gemm_split_tn_partial_floats(M, K, N) floats.
size_t gemm_split_tn_partial_floats(int64_t M, int64_t K, int N);
int gemm_split_tn(const void *a, const void *b_units, int b_ld, float *c, int ldc, int64_t M, int64_t K, int N,
                  float *partials, size_t partial_floats, hipStream_t st);

// ---------------------------------------------------------------------------------------------
// Event timing of launches (api.hip): timing_open records an event on the stream the work is about to be launched
// on and returns a handle (-1 when the part is not being timed); timing_close records the closing event.
// `part` is a gcn_timed_part of include/gcn355_debug.h.
int timing_open(int part, int width, hipStream_t st);
void timing_close(int handle, hipStream_t st);
bool timing_enabled();
enum {
    kTimeAggregate = GCN_TIME_AGGREGATE, kTimeGather = GCN_TIME_GATHER, kTimeTiles = GCN_TIME_TILES,
    kTimePlanes = GCN_TIME_PLANES, kTimeJoin = GCN_TIME_JOIN, kTimeGemmNN = GCN_TIME_GEMM_NN,
    kTimeGemmTN = GCN_TIME_GEMM_TN, kTimeGemmNT = GCN_TIME_GEMM_NT, kTimeLoss = GCN_TIME_LOSS,
    kTimeSageGather = GCN_TIME_SAGE_GATHER
};

}  // namespace gcn

// C ABI of libgcn355.so and the host-side step scheduler: which kernel runs when, on which buffer.
// The arithmetic lives in the kernels; this file only validates arguments, carves the caller's
// workspaces and enqueues launches (layer rule and training scheme: Sections 4.1 and 3.2).
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <string>

#include "common.hpp"
#include "graph_object.hpp"

namespace gcn {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

// ------------------------------------------------------------------------------------------- tunables
namespace {
std::mutex g_knob_mutex;
std::vector<std::pair<std::string, int64_t>> g_knobs;
}  // namespace

int64_t tunable(const char *name, int64_t fallback) {
    std::lock_guard<std::mutex> lk(g_knob_mutex);
    for (auto &k : g_knobs)
        if (k.first == name) return k.second;
    return fallback;
}

// ------------------------------------------------------------------------------------------- timing
namespace {
struct TimedLaunch {
    int part, width;
    hipEvent_t start, stop;
    bool closed;
};
std::mutex g_tmutex;
int g_timing = 0;   // 0 off, 1 whole aggregations (and the GraphSAGE gather), 2 also their parts and the dense products
std::vector<TimedLaunch> g_launches;
std::vector<std::pair<hipEvent_t, hipEvent_t>> g_free_events;
}  // namespace

int timing_open(int part, int width, hipStream_t st) {
    std::lock_guard<std::mutex> lk(g_tmutex);
    const int level = (part == kTimeAggregate || part == kTimeSageGather) ? 1 : 2;
    if (g_timing < level) return -1;
    std::pair<hipEvent_t, hipEvent_t> ev;
    if (!g_free_events.empty()) {
        ev = g_free_events.back();
        g_free_events.pop_back();
    } else {
        if (hipEventCreate(&ev.first) != hipSuccess) return -1;
        if (hipEventCreate(&ev.second) != hipSuccess) {
            (void)hipEventDestroy(ev.first);
            return -1;
        }
    }
    if (hipEventRecord(ev.first, st) != hipSuccess) {
        g_free_events.push_back(ev);
        return -1;
    }
    g_launches.push_back({part, width, ev.first, ev.second, false});
    return (int)g_launches.size() - 1;
}

void timing_close(int handle, hipStream_t st) {
    std::lock_guard<std::mutex> lk(g_tmutex);
    if (handle < 0 || handle >= (int)g_launches.size() || g_launches[handle].closed) return;
    if (hipEventRecord(g_launches[handle].stop, st) == hipSuccess) g_launches[handle].closed = true;
}

bool timing_enabled() {
    std::lock_guard<std::mutex> lk(g_tmutex);
    return g_timing != 0;
}

}  // namespace gcn

using namespace gcn;

// ------------------------------------------------------------------------------------------- objects
struct Layer {
    int d_in, d_out, ld_in, ld_out;
    float *w;    // ld_in x ld_out
    float *dw;   // ld_in x ld_out
    // the next four hold the model's storage type (float or bfloat16); the logits are always float
    void *t;     // (n + 1) x ld_out : D^-1/2 (H_{l-1} W_l), row n zero
    void *h;     // n x ld_out : H_l (l < L) or the logits (l = L)
    void *dzs;   // (n + 1) x ld_out : D^-1/2 dLoss/dZ_l, row n zero
    void *g;     // n x ld_out : A_hat dLoss/dZ_l
    float *am;   // Adam first moment, ld_in x ld_out
    float *av;   // Adam second moment
    void *wb;    // bfloat16 mode: W as bfloat16, ld_in x ld_out
    void *wbt;   // bfloat16 mode: W^T as bfloat16, ld_out x ld_in
};

struct gcn_model {
    const gcn_graph *g = nullptr;
    int L = 0;
    int dtype = GCN_F32;
    std::vector<Layer> layers;
    float p = 0.f;
    uint64_t seed = 0, epoch = 0;
    int64_t adam_steps = 0;
    float *partials = nullptr;
    size_t partial_floats = 0;
    float *tile_sums = nullptr;     // n x widest aggregated matrix: the tile product's output when it runs beside the gather
    float *gather_sums = nullptr;   // the same for the gather's plain sums (bfloat16 models only)
    float *chunk_sums = nullptr;    // chunks x widest: sums of the chunks of split rows
    double *loss_part = nullptr;
    long long *corr_part = nullptr;
    float *result = nullptr;        // [0] loss [1] accuracy
    long long *result_correct = nullptr;
    bool have_forward = false, have_loss = false, have_backward = false, trained_forward = false;
    bool dz_units_ready = false;   // gcn_loss_acc left dLoss/dlogits in the tile product's order as well
    // Layer 1 in aggregate-first form: P = A_hat X is computed once (X never changes), then
    // Z_1 = P W_1 and dW_1 = P^T dZ_1 need no aggregation at all.
    bool l1_cached = false;
    void *pax = nullptr;  // (n + 1) x ldf, storage type
    void *xs = nullptr;   // (n + 1) x ldf: D^-1/2 X, only used while P is built
    // Layer 1's feature transform on the bfloat16 matrix instruction (float32 models): the constant left operand
    // (X, or P) is packed once, W_1^T before each product.
    bool l1_split = false;
    void *sp_a = nullptr;    // packed left operand [n x ld_in]
    void *sp_wt = nullptr;   // packed right operand [ld_out x ld_in]
    void *sp_at = nullptr;   // the same matrix as sp_a transposed, packed left [ld_in x n] (weight gradient)
    void *sp_gu = nullptr;   // the weight gradient's right operand [n x ld_out] in the tile product's order
};

namespace {

uint64_t host_mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

bool aligned256(const void *p) { return ((uintptr_t)p & 255u) == 0; }

// floats of the tile product's buffer for one aggregation of `cols` columns: the n x cols sums, then the partial
// sums (blocks of kTileRows x cols), then the input split into bfloat16 planes (sized for float32 input, the larger case)
size_t tile_partial_offset(const gcn_graph *g, int cols) { return (size_t)g->n * (size_t)cols; }
size_t tile_planes_offset(const gcn_graph *g, int cols) {
    const size_t floats = ((size_t)g->n + (size_t)g->tiles.n_slots * kTileRows) * (size_t)cols;
    return (floats + 63) & ~(size_t)63;   // 256-byte aligned when the buffer is
}
size_t tile_sum_floats(const gcn_graph *g, int cols) {
    return tile_planes_offset(g, cols) + tiles_plane_bytes(g->n, cols, GCN_F32) / sizeof(float);
}

// floats for the chunk sums of one aggregation of `cols` columns over either form of the pattern
size_t chunk_sum_floats(const gcn_graph *g, int cols) {
    int64_t chunks = g->rows.n_chunks > g->res_rows.n_chunks ? g->rows.n_chunks : g->res_rows.n_chunks;
    if (g->bwd_rows.n_chunks > chunks) chunks = g->bwd_rows.n_chunks;
    return (size_t)chunks * (size_t)cols;
}

// tile_sums: tile_sum_floats(g, cols) floats for the tile product (its output when it runs beside the gather kernel,
// and the partial sums of row blocks whose tiles were cut into runs);
// gather_sums: the same again for the gather kernel's plain sums when the output is bfloat16 (else null)
SpmmArgs spmm_args(const gcn_graph *g, const void *t, int t_dtype, int ld_t, void *out, int out_dtype, int ld_out,
                   int cols, int width, int epilogue, float *tile_sums, float *chunk_sums,
                   float *gather_sums = nullptr, bool rows_zero_outside_mask = false) {
    SpmmArgs a{};
    // The dense-tile form: float32 matrices either way (side by side or one after the other); bfloat16 inputs
    // side by side only, and with a bfloat16 output only with a buffer for the gather's float32 sums.  Everything
    // else gathers over the whole pattern.
    const bool side_by_side = tile_sums && g->side && tunable("spmm_overlap", 1) != 0;
    const bool tiles = g->use_tiles && tunable("spmm_tiles", -1) != 0 && cols <= 256 &&
                       ((t_dtype == GCN_F32 && out_dtype == GCN_F32) ||
                        (t_dtype == GCN_BF16 && side_by_side && (out_dtype == GCN_F32 || gather_sums)));
    // rows_zero_outside_mask: the caller vouches that the input's rows of vertices outside the train mask are zero;
    // then the pattern without their columns gives the same sums (it was cut from the pattern of the default form)
    const bool masked = rows_zero_outside_mask && g->use_bwd && tiles == g->use_tiles;
    const PrepBuffers &pb = masked ? g->bwd : (tiles ? g->res : g->pb);
    a.rowptr = pb.rowptr;
    a.col = pb.col;
    a.perm = pb.perm;
    a.dinv = g->pb.dinv;
    a.segoff = pb.segoff;
    a.prow = pb.prow;

    a.n = g->n;
    a.spread = g->tiles_searched && g->nnz_dense * 16 < g->E;
    const gcn_graph::RowClasses &rc = masked ? g->bwd_rows : (tiles ? g->res_rows : g->rows);
    a.phased_w = rc.phased_w;
    a.phased_r = rc.phased_r;
    a.n_heavy = rc.n_heavy;
    a.n_light = rc.n_light;
    a.n_split = rc.n_split;
    a.n_chunks = rc.n_chunks;
    a.xcd_start = pb.xcd_start;
    a.xcd_rows_max = rc.xcd_rows_max;
    a.chunk_off = pb.chunk_off;
    a.chunk_srow = pb.chunk_srow;
    a.chunk_sums = chunk_sums;
    if (tiles) {
        a.tile_ptr = g->tiles.tile_ptr;
        a.tile_col = g->tiles.tile_col;
        a.bits = g->tiles.bits;
        a.tile_items = g->tiles.items;
        a.n_items = g->tiles.n_items;
        a.tile_folds = g->tiles.folds;
        a.n_folds = g->tiles.n_folds;
        a.n_slots = g->tiles.n_slots;
        // the partial sums of row blocks whose tiles were cut into runs follow the n x cols sums in the same buffer
        // (the buffer was sized for the widest aggregation, so this one's parts fit)
        a.tile_partial = tile_sums ? tile_sums + tile_partial_offset(g, cols) : nullptr;
        a.tile_planes = tile_sums ? tile_sums + tile_planes_offset(g, cols) : nullptr;
        if (tile_sums && g->side) {
            a.gather_sums = gather_sums;
            a.tile_sums = tile_sums;
            a.side = g->side;
            a.ev_fork = g->ev_fork;
            a.ev_join = g->ev_join;
        }
    }
    a.t = t;
    a.t_dtype = t_dtype;
    a.ld_t = ld_t;
    a.out = out;
    a.out_dtype = out_dtype;
    a.ld_out = ld_out;
    a.cols = cols;
    a.width = width;
    a.epilogue = epilogue;
    a.drop_threshold = 0u;
    a.keep_scale = 1.0f;
    a.drop_key = 0ull;
    return a;
}

void carve_graph(Carver &c, gcn_graph &g) {
    const int64_t n = g.n, cap = g.nnz_in + n;
    g.pb.rowptr = c.take<int64_t>(n + 1);
    g.pb.col = c.take<int32_t>(cap + kColSlack);
    g.pb.deg = c.take<int32_t>(n);
    g.pb.dinv = c.take<float>(n);
    g.pb.perm = c.take<int32_t>(n);
    g.pb.scratch = c.take<int32_t>(cap);
    g.pb.heavy = c.take<int32_t>(n);
    g.pb.hpos = c.take<int64_t>(n + 1);
    g.pb.lpos = c.take<int64_t>(n + 1);
    g.pb.split_cap = cap / kSplitDegree + 1;
    g.pb.chunk_cap = cap / kChunk + g.pb.split_cap + 1;
    g.pb.split_cnt = c.take<int32_t>(g.pb.split_cap);
    g.pb.chunk_off = c.take<int64_t>(g.pb.split_cap + 1);
    g.pb.chunk_srow = c.take<int32_t>(g.pb.chunk_cap);
    g.pb.xcd_start = c.take<int32_t>(16);
    const bool phased = phased_possible(n);   // (a null pointer says nothing here: a measuring Carver returns null)
    g.pb.segoff = phased ? c.take<int32_t>((size_t)n * (kColBlocks + 1)) : nullptr;
    const size_t prow_ints = (size_t)kXcds * (kPhasedMaxRows + 8);
    g.pb.prow = phased ? c.take<int32_t>(prow_ints) : nullptr;
    g.pb.row_start = c.take<int32_t>(16);
    g.pb.blocksum = c.take<int64_t>(scan_blocks(n > g.pb.split_cap ? n : g.pb.split_cap));
    g.pb.flags = c.take<int32_t>(16);
    TileBuffers &tb = g.tiles;
    tb.n_rb = (n + kTileRows - 1) / kTileRows;
    tb.capacity = (int64_t)tiles_capacity(cap);
    tb.tile_cnt = c.take<int32_t>(tb.n_rb);
    tb.tile_ptr = c.take<int64_t>(tb.n_rb + 1);
    tb.tile_col = c.take<int32_t>(tb.capacity);
    tb.tile_rt = c.take<int32_t>(tb.capacity);
    tb.bits = c.take<uint32_t>((size_t)tb.capacity * kTileRows);
    tb.totals = c.take<unsigned long long>(2);
    tb.item_capacity = tiles_item_capacity(tb.n_rb, tb.capacity);
    tb.items = c.take<int32_t>(tb.item_capacity * 4);
    tb.folds = c.take<int32_t>((size_t)tb.n_rb * 4);
    g.res = g.pb;   // shares dinv and the creation-time scratch arrays; its own pattern and schedule follow
    g.res.rowptr = c.take<int64_t>(n + 1);
    g.res.col = c.take<int32_t>(cap + kColSlack);
    g.res.deg = c.take<int32_t>(n);
    g.res.perm = c.take<int32_t>(n);
    g.res.split_cnt = c.take<int32_t>(g.pb.split_cap);
    g.res.chunk_off = c.take<int64_t>(g.pb.split_cap + 1);
    g.res.chunk_srow = c.take<int32_t>(g.pb.chunk_cap);
    g.res.xcd_start = c.take<int32_t>(16);
    g.res.segoff = phased ? c.take<int32_t>((size_t)n * (kColBlocks + 1)) : nullptr;
    g.res.prow = phased ? c.take<int32_t>(prow_ints) : nullptr;
    g.res.row_start = c.take<int32_t>(16);
    g.res.flags = c.take<int32_t>(16);
    g.bwd = g.pb;   // as the residual pattern: its own pattern and schedule, the rest shared
    g.bwd.rowptr = c.take<int64_t>(n + 1);
    g.bwd.col = c.take<int32_t>(cap + kColSlack);
    g.bwd.deg = c.take<int32_t>(n);
    g.bwd.perm = c.take<int32_t>(n);
    g.bwd.split_cnt = c.take<int32_t>(g.pb.split_cap);
    g.bwd.chunk_off = c.take<int64_t>(g.pb.split_cap + 1);
    g.bwd.chunk_srow = c.take<int32_t>(g.pb.chunk_cap);
    g.bwd.xcd_start = c.take<int32_t>(16);
    g.bwd.segoff = phased ? c.take<int32_t>((size_t)n * (kColBlocks + 1)) : nullptr;
    g.bwd.prow = phased ? c.take<int32_t>(prow_ints) : nullptr;
    g.bwd.row_start = c.take<int32_t>(16);
    g.bwd.flags = c.take<int32_t>(16);
    g.x = c.take<char>((size_t)(n + 1) * g.ldf * (g.store_dtype == GCN_BF16 ? 2 : 4));
    g.labels = c.take<int32_t>(n);
    g.mask = c.take<uint8_t>(n);
}

void carve_model(Carver &c, gcn_model &m) {
    const int64_t n = m.g->n;
    size_t pf = 0;
    for (auto &ly : m.layers) {
        ly.w = c.take<float>((size_t)ly.ld_in * ly.ld_out);
        ly.dw = c.take<float>((size_t)ly.ld_in * ly.ld_out);
        ly.am = c.take<float>((size_t)ly.ld_in * ly.ld_out);
        ly.av = c.take<float>((size_t)ly.ld_in * ly.ld_out);
        const size_t es = m.dtype == GCN_BF16 ? 2 : 4;
        const size_t act = (size_t)(n + 1) * ly.ld_out;
        ly.t = c.take<char>(act * es);
        ly.h = c.take<char>(act * 4);          // float-sized even in bfloat16 mode: the last layer's logits are float
        ly.dzs = c.take<char>(act * es);
        ly.g = c.take<char>(act * es);
        ly.wb = ly.wbt = nullptr;
        if (m.dtype == GCN_BF16) {
            ly.wb = c.take<char>((size_t)ly.ld_in * ly.ld_out * 2);
            ly.wbt = c.take<char>((size_t)ly.ld_in * ly.ld_out * 2);
        }
        size_t need = m.dtype == GCN_BF16 ? gemm_bf16_tn_partial_floats(n, ly.ld_in, ly.ld_out)
                                          : gemm_tn_partial_floats(n, ly.ld_in, ly.ld_out);
        if (need > pf) pf = need;
    }
    if (m.l1_cached) {
        const size_t es = m.dtype == GCN_BF16 ? 2 : 4;
        m.pax = c.take<char>((size_t)(n + 1) * m.g->ldf * es);
        m.xs = c.take<char>((size_t)(n + 1) * m.g->ldf * es);
    }
    if (m.l1_split) {
        const Layer &l1 = m.layers[0];
        m.sp_a = c.take<char>(packed_bytes(n, l1.ld_in, true));
        m.sp_wt = c.take<char>(packed_bytes(l1.ld_out, l1.ld_in, false));
        // The weight gradient the same way only when layer 1 works from the cached A_hat X ("gemm_split_tn", default
        // 1): there dZ_1 comes out of the product above it already in the order the right operand is read in, and an
        // epoch gains 4 % (1,946 against 1,875 epochs/s on the Reddit-shaped partition).  Behind an aggregation the
        // product itself is as much faster (83 against 91 us), but the epoch is not (938 against 944 epochs/s; the
        // clock the chip settles to under the loop drops with every product moved to the bfloat16 instruction).
        if (m.l1_cached && tunable("gemm_split_tn", 1) != 0) {
            m.sp_at = c.take<char>(packed_bytes(l1.ld_in, n, true));
            m.sp_gu = c.take<char>(tiles_plane_bytes(n, l1.ld_out, GCN_F32));
            const size_t need = gemm_split_tn_partial_floats(l1.ld_in, n, l1.ld_out);
            if (need > pf) pf = need;
        }
    }
    int widest = 0;   // columns of the widest single aggregation launch
    for (auto &ly : m.layers) widest = ly.ld_out > widest ? ly.ld_out : widest;
    if (m.l1_cached) {   // P = A_hat X is built in slabs of 256 (float32) or 512 (bfloat16) columns
        const int slab_max = m.dtype == GCN_BF16 ? 512 : 256;
        const int slab = slab_max < m.g->ldf ? slab_max : m.g->ldf;
        widest = slab > widest ? slab : widest;
    }
    m.tile_sums = m.g->use_tiles ? c.take<float>(tile_sum_floats(m.g, widest)) : nullptr;
    m.gather_sums = (m.g->use_tiles && m.dtype == GCN_BF16) ? c.take<float>((size_t)n * widest) : nullptr;
    m.chunk_sums = c.take<float>(chunk_sum_floats(m.g, widest));
    m.partial_floats = pf;
    m.partials = c.take<float>(pf);
    m.loss_part = c.take<double>(kLossBlocks);
    m.corr_part = c.take<long long>(kLossBlocks);
    m.result = c.take<float>(4);
    m.result_correct = c.take<long long>(2);
}

// "cache_ax" knob: 0 = never, 1 = when the input is not wider than the first hidden layer (default), 2 = always.
// Needs at least two layers (the one-layer model's output are float logits straight from the aggregation).
bool want_l1_cached(int32_t n_layers, const int32_t *dims) {
    const int64_t knob = tunable("cache_ax", 1);
    if (n_layers < 2 || knob <= 0) return false;
    return knob >= 2 || dims[0] <= dims[1];
}

// "gemm_split" knob: float32 models run layer 1's feature transform on the bfloat16 matrix instruction with
// three-plane operands: 0 = never, 1 = when the input is at least 256 wide (default), 2 = always.  (The product
// loads two blocks of 32 of the shared index ahead; over the four blocks of a 128-wide input that does not pay:
// 128-128-40 on the 100,000-vertex Chung-Lu graph 2,086 against 2,136 epochs/s, 3,353 against 3,361 from the
// cached A_hat X; the 602-wide Reddit shapes gain 2 to 8 %.)
bool want_l1_split(int dtype, int d_in) {
    const int64_t knob = tunable("gemm_split", 1);
    return dtype == GCN_F32 && (knob >= 2 || (knob == 1 && d_in >= 256));
}

// Layer widths: 1..16 layers; the input may be up to 4096 wide; hidden and output widths are limited to what one
// aggregation launch covers with a wave per row (64 lanes x 16 bytes): 256 columns in float32, 512 in bfloat16.
int check_dims(int32_t n_layers, const int32_t *dims, int dtype) {
    if (n_layers < 1 || n_layers > 16 || !dims) return GCN_EINVAL;
    if (dims[0] < 1 || dims[0] > 4096) return GCN_EINVAL;
    const int max_w = dtype == GCN_BF16 ? 512 : 256;
    for (int l = 1; l <= n_layers; ++l)
        if (dims[l] < 1 || dims[l] > max_w) return GCN_EINVAL;
    return GCN_OK;
}

}  // namespace

// ------------------------------------------------------------------------------------------- C ABI
extern "C" {

const char *gcn_last_error(void) { return g_err; }

int gcn_graph_workspace_bytes(int64_t n, int64_t nnz_in, int32_t f, int store_dtype, size_t *bytes) {
    if (!bytes || n <= 0 || n >= 0x7ffffff0 || nnz_in < 0 || f < 1 ||
        (store_dtype != GCN_F32 && store_dtype != GCN_BF16)) {
        set_error("gcn_graph_workspace_bytes: bad argument");
        return GCN_EINVAL;
    }
    gcn_graph g;
    g.store_dtype = store_dtype;
    g.n = n;
    g.nnz_in = nnz_in;
    g.f = f;
    g.ldf = padded_width(f);
    Carver c(nullptr);
    carve_graph(c, g);
    *bytes = c.bytes();
    return GCN_OK;
}

int gcn_graph_create(gcn_graph **out, int64_t n, int64_t nnz_in, const int64_t *rowptr, const int32_t *col,
                     const float *feat, int32_t f, int store_dtype, const int32_t *labels,
                     const uint8_t *train_mask, int32_t n_classes, void *workspace, size_t workspace_bytes,
                     void *stream) {
    if (out) *out = nullptr;
    if (!out || !rowptr || (!col && nnz_in > 0) || !feat || !labels || !train_mask || n <= 0 || n >= 0x7ffffff0 ||
        nnz_in < 0 || f < 1 || n_classes < 1) {
        set_error("gcn_graph_create: null pointer or bad size");
        return GCN_EINVAL;
    }
    size_t need = 0;
    int rc = gcn_graph_workspace_bytes(n, nnz_in, f, store_dtype, &need);
    if (rc) return rc;
    if (!workspace || !aligned256(workspace) || workspace_bytes < need) {
        set_error("gcn_graph_create: workspace missing, misaligned or smaller than %zu bytes", need);
        return GCN_EWORKSPACE;
    }
    hipStream_t st = (hipStream_t)stream;
    gcn_graph *g = new (std::nothrow) gcn_graph;
    if (!g) {
        set_error("out of host memory");
        return GCN_EINVAL;
    }
    g->n = n;
    g->nnz_in = nnz_in;
    g->f = f;
    g->ldf = padded_width(f);
    g->n_classes = n_classes;
    g->store_dtype = store_dtype;
    Carver c(workspace);
    carve_graph(c, *g);   // uses store_dtype
    if (c.bytes() != need) {   // the measuring pass and this one must lay out the same buffers
        set_error("gcn_graph_create: internal layout mismatch (%zu bytes carved, %zu measured)", c.bytes(), need);
        delete g;
        return GCN_EINVAL;
    }
    int32_t flags[16];

#define FAIL_IF(expr)            \
    do {                         \
        int rc_ = (expr);        \
        if (rc_) {               \
            delete g;            \
            return rc_;          \
        }                        \
    } while (0)
#define HIP_OR_FAIL(call)                                                                       \
    do {                                                                                        \
        hipError_t e_ = (call);                                                                 \
        if (e_ != hipSuccess) {                                                                 \
            set_error("%s failed: %s", #call, hipGetErrorString(e_));                           \
            delete g;                                                                           \
            return GCN_EHIP;                                                                    \
        }                                                                                       \
    } while (0)

    FAIL_IF(fill_zero(g->pb.flags, 16 * sizeof(int32_t), st));
    FAIL_IF(prep_validate(n, nnz_in, rowptr, col, g->pb.flags, st));
    FAIL_IF(prep_labels_mask(n, labels, train_mask, n_classes, g->labels, g->mask, g->pb.flags, st));
    HIP_OR_FAIL(hipMemcpyAsync(flags, g->pb.flags, sizeof(flags), hipMemcpyDeviceToHost, st));
    HIP_OR_FAIL(hipStreamSynchronize(st));
    if (flags[0]) {
        set_error("gcn_graph_create: invalid CSR (%s)", (flags[0] & 1) ? "rowptr" : "column index out of range");
        delete g;
        return GCN_EGRAPH;
    }
    if (flags[1]) {
        set_error("gcn_graph_create: a label is outside [0, %d)", n_classes);
        delete g;
        return GCN_ELABEL;
    }
    if (flags[2] <= 0) {
        set_error("gcn_graph_create: the train mask is empty");
        delete g;
        return GCN_EINVAL;
    }
    g->n_train = flags[2];

    FAIL_IF(prep_canonical(n, nnz_in, rowptr, col, g->pb, st));
    FAIL_IF(prep_schedule(n, g->pb, st));
    const size_t x_es = store_dtype == GCN_BF16 ? 2 : 4;
    FAIL_IF(pad_rows(feat, n, f, g->x, store_dtype, g->ldf, nullptr, st));
    FAIL_IF(fill_zero((char *)g->x + (size_t)n * g->ldf * x_es, (size_t)g->ldf * x_es, st));
    int64_t ends[1];
    HIP_OR_FAIL(hipMemcpyAsync(flags, g->pb.flags, sizeof(flags), hipMemcpyDeviceToHost, st));
    HIP_OR_FAIL(hipMemcpyAsync(&ends[0], g->pb.rowptr + n, sizeof(int64_t), hipMemcpyDeviceToHost, st));
    HIP_OR_FAIL(hipStreamSynchronize(st));
    if (flags[0] & 4) {
        set_error("gcn_graph_create: the adjacency pattern is not symmetric");
        delete g;
        return GCN_EGRAPH;
    }
    g->E = ends[0];
    g->max_deg = flags[3];
    auto read_classes = [&](const PrepBuffers &pb, const int32_t *fl, gcn_graph::RowClasses &rc) -> hipError_t {
        rc.n_heavy = fl[4];
        rc.n_light = fl[5];
        rc.n_split = n - rc.n_heavy - rc.n_light;
        int32_t starts[kXcds + 1];
        hipError_t e = hipMemcpyAsync(&rc.n_chunks, pb.chunk_off + pb.split_cap, sizeof(int64_t), hipMemcpyDeviceToHost, st);
        if (e == hipSuccess) e = hipMemcpyAsync(starts, pb.xcd_start, sizeof(starts), hipMemcpyDeviceToHost, st);
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        rc.xcd_rows_max = 0;
        if (e == hipSuccess)
            for (int x = 0; x < kXcds; ++x)
                if (starts[x + 1] - starts[x] > rc.xcd_rows_max) rc.xcd_rows_max = starts[x + 1] - starts[x];
        // the phased schedule: equal entries per XCD; available when the longest of its row ranges fits
        rc.phased_w = rc.phased_r = 0;
        if (e == hipSuccess && pb.prow) {
            e = hipMemcpyAsync(starts, pb.row_start, sizeof(starts), hipMemcpyDeviceToHost, st);
            if (e == hipSuccess) e = hipStreamSynchronize(st);
            int64_t longest = 0;
            if (e == hipSuccess)
                for (int x = 0; x < kXcds; ++x)
                    if (starts[x + 1] - starts[x] > longest) longest = starts[x + 1] - starts[x];
            int w = 0, r = 0;
            if (e == hipSuccess && phased_shape(longest, &w, &r)) {
                if (prep_balance_rows(n, pb.deg, pb.row_start, w, r, pb.prow, st) == GCN_OK) {
                    rc.phased_w = w;
                    rc.phased_r = r;
                }
            }
        }
        return e;
    };
    HIP_OR_FAIL(read_classes(g->pb, flags, g->rows));

    // Dense tiles: select, then decide.  Knobs read here: "tile_min_entries" (default kTileMinEntriesDefault of the 4096 places of a tile), "spmm_tiles"
    // (-1: use the tiles when they hold at least a quarter of the entries, 0: never build, 1: whenever there is one).
    const int64_t tiles_knob = tunable("spmm_tiles", -1);
    if (tiles_knob != 0) {
        int64_t me = tunable("tile_min_entries", kTileMinEntriesDefault);
        if (me < kTileMinEntriesFloor) me = kTileMinEntriesFloor;
        if (me > kTileRows * 32) me = kTileRows * 32;
        FAIL_IF(tiles_select(n, g->pb.rowptr, g->pb.col, (int)me, g->tiles, g->pb.blocksum, st));
        unsigned long long dense = 0;
        HIP_OR_FAIL(hipMemcpyAsync(&g->n_tiles, g->tiles.tile_ptr + g->tiles.n_rb, sizeof(int64_t),
                                   hipMemcpyDeviceToHost, st));
        HIP_OR_FAIL(hipMemcpyAsync(&dense, g->tiles.totals, sizeof(dense), hipMemcpyDeviceToHost, st));
        HIP_OR_FAIL(hipStreamSynchronize(st));
        g->nnz_dense = (int64_t)dense;
        g->tiles_searched = true;
        if (g->n_tiles > g->tiles.capacity) {   // cannot happen: every tile holds >= kTileMinEntriesFloor entries
            set_error("gcn_graph_create: dense tile count %lld exceeds capacity", (long long)g->n_tiles);
            delete g;
            return GCN_EINVAL;
        }
        g->use_tiles = g->n_tiles > 0 && (tiles_knob > 0 || g->nnz_dense * 4 >= g->E);
        if (g->use_tiles) {
            FAIL_IF(tiles_build(n, g->pb.rowptr, g->pb.col, g->n_tiles, g->tiles, g->res, st));
            std::vector<int64_t> tile_ptr((size_t)g->tiles.n_rb + 1);
            HIP_OR_FAIL(hipMemcpyAsync(tile_ptr.data(), g->tiles.tile_ptr, tile_ptr.size() * sizeof(int64_t),
                                       hipMemcpyDeviceToHost, st));
            HIP_OR_FAIL(hipStreamSynchronize(st));
            FAIL_IF(tiles_plan(tile_ptr, g->tiles, st));
            FAIL_IF(fill_zero(g->res.flags, 16 * sizeof(int32_t), st));
            FAIL_IF(prep_schedule(n, g->res, st));
            HIP_OR_FAIL(hipMemcpyAsync(flags, g->res.flags, sizeof(flags), hipMemcpyDeviceToHost, st));
            HIP_OR_FAIL(hipStreamSynchronize(st));
            HIP_OR_FAIL(read_classes(g->res, flags, g->res_rows));
            HIP_OR_FAIL(hipStreamCreateWithFlags(&g->side, hipStreamNonBlocking));   // default priority
            HIP_OR_FAIL(hipEventCreateWithFlags(&g->ev_fork, hipEventDisableTiming));
            HIP_OR_FAIL(hipEventCreateWithFlags(&g->ev_join, hipEventDisableTiming));
            HIP_OR_FAIL(hipEventCreateWithFlags(&g->ev_aux, hipEventDisableTiming));
        }
    }
    // The last layer's backward aggregation reads dLoss/dlogits, whose rows outside the train mask are zero: a
    // pattern without those columns, when that drops at least a fifth of the vertices' columns.
    if (g->n_train * 5 <= n * 4 && tunable("spmm_masked", 1) != 0) {
        const PrepBuffers &src = g->use_tiles ? g->res : g->pb;
        FAIL_IF(prep_keep_columns(n, src, g->mask, g->bwd, st));
        FAIL_IF(fill_zero(g->bwd.flags, 16 * sizeof(int32_t), st));
        FAIL_IF(prep_schedule(n, g->bwd, st));
        HIP_OR_FAIL(hipMemcpyAsync(flags, g->bwd.flags, sizeof(flags), hipMemcpyDeviceToHost, st));
        HIP_OR_FAIL(hipMemcpyAsync(&g->bwd_nnz, g->bwd.rowptr + n, sizeof(int64_t), hipMemcpyDeviceToHost, st));
        HIP_OR_FAIL(hipStreamSynchronize(st));
        HIP_OR_FAIL(read_classes(g->bwd, flags, g->bwd_rows));
        g->use_bwd = true;
    }
#undef FAIL_IF
#undef HIP_OR_FAIL
    *out = g;
    return GCN_OK;
}

int gcn_graph_get_masked_pattern(const gcn_graph *g, int64_t *rowptr, int32_t *col, int64_t *nnz, void *stream) {
    if (!g) {
        set_error("gcn_graph_get_masked_pattern: null graph");
        return GCN_EINVAL;
    }
    if (!g->use_bwd) {
        set_error("gcn_graph_get_masked_pattern: this graph has none");
        return GCN_EINVAL;
    }
    hipStream_t st = (hipStream_t)stream;
    if (nnz) *nnz = g->bwd_nnz;
    hipError_t e = hipSuccess;
    if (rowptr) e = hipMemcpyAsync(rowptr, g->bwd.rowptr, (size_t)(g->n + 1) * sizeof(int64_t), hipMemcpyDeviceToDevice, st);
    if (e == hipSuccess && col && g->bwd_nnz > 0)
        e = hipMemcpyAsync(col, g->bwd.col, (size_t)g->bwd_nnz * sizeof(int32_t), hipMemcpyDeviceToDevice, st);
    if (e != hipSuccess) {
        set_error("gcn_graph_get_masked_pattern: copy failed: %s", hipGetErrorString(e));
        return GCN_EHIP;
    }
    return GCN_OK;
}

int gcn_graph_destroy(gcn_graph *g) {
    delete g;
    return GCN_OK;
}

int gcn_graph_info(const gcn_graph *g, int64_t *n, int64_t *nnz, int64_t *n_train, int32_t *max_degree) {
    if (!g) {
        set_error("gcn_graph_info: null graph");
        return GCN_EINVAL;
    }
    if (n) *n = g->n;
    if (nnz) *nnz = g->E;
    if (n_train) *n_train = g->n_train;
    if (max_degree) *max_degree = g->max_deg;
    return GCN_OK;
}

int gcn_graph_tile_info(const gcn_graph *g, int64_t *n_tiles, int64_t *nnz_dense, int32_t *in_use) {
    if (!g) {
        set_error("gcn_graph_tile_info: null graph");
        return GCN_EINVAL;
    }
    if (n_tiles) *n_tiles = g->n_tiles;
    if (nnz_dense) *nnz_dense = g->nnz_dense;
    if (in_use) *in_use = g->use_tiles ? 1 : 0;
    return GCN_OK;
}

int gcn_graph_get_tiles(const gcn_graph *g, int64_t *tile_ptr, int32_t *tile_col, uint32_t *bits,
                        int64_t *res_rowptr, int32_t *res_col, int64_t *res_nnz, void *stream) {
    if (!g) {
        set_error("gcn_graph_get_tiles: null graph");
        return GCN_EINVAL;
    }
    if (!g->use_tiles) {
        set_error("gcn_graph_get_tiles: this graph does not use dense tiles");
        return GCN_EINVAL;
    }
    hipStream_t st = (hipStream_t)stream;
    const int64_t res_E = g->E - g->nnz_dense;
    if (res_nnz) *res_nnz = res_E;
    if (tile_ptr)
        GCN_HIP(hipMemcpyAsync(tile_ptr, g->tiles.tile_ptr, (g->tiles.n_rb + 1) * sizeof(int64_t),
                               hipMemcpyDeviceToDevice, st));
    if (tile_col)
        GCN_HIP(hipMemcpyAsync(tile_col, g->tiles.tile_col, g->n_tiles * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
    if (bits)
        GCN_HIP(hipMemcpyAsync(bits, g->tiles.bits, g->n_tiles * kTileRows * sizeof(uint32_t), hipMemcpyDeviceToDevice,
                               st));
    if (res_rowptr)
        GCN_HIP(hipMemcpyAsync(res_rowptr, g->res.rowptr, (g->n + 1) * sizeof(int64_t), hipMemcpyDeviceToDevice, st));
    if (res_col && res_E > 0)
        GCN_HIP(hipMemcpyAsync(res_col, g->res.col, res_E * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
    return GCN_OK;
}

int gcn_graph_get_csr(const gcn_graph *g, int64_t *rowptr, int32_t *col, int32_t *deg, float *dinv, void *stream) {
    if (!g) {
        set_error("gcn_graph_get_csr: null graph");
        return GCN_EINVAL;
    }
    hipStream_t st = (hipStream_t)stream;
    if (rowptr) GCN_HIP(hipMemcpyAsync(rowptr, g->pb.rowptr, (g->n + 1) * sizeof(int64_t), hipMemcpyDeviceToDevice, st));
    if (col) GCN_HIP(hipMemcpyAsync(col, g->pb.col, g->E * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
    if (deg) GCN_HIP(hipMemcpyAsync(deg, g->pb.deg, g->n * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
    if (dinv) GCN_HIP(hipMemcpyAsync(dinv, g->pb.dinv, g->n * sizeof(float), hipMemcpyDeviceToDevice, st));
    return GCN_OK;
}

int gcn_aggregate_workspace_bytes(const gcn_graph *g, int32_t width, int dtype, size_t *bytes) {
    if (!g || !bytes || width < 1 || (dtype != GCN_F32 && dtype != GCN_BF16) ||
        width > (dtype == GCN_BF16 ? 512 : 256)) {
        set_error("gcn_aggregate_workspace_bytes: bad argument");
        return GCN_EINVAL;
    }
    Carver c(nullptr);
    const int ld = padded_width(width);
    c.take<float>((size_t)(g->n + 1) * ld);
    c.take<float>((size_t)(g->n + 1) * ld);
    c.take<float>(tile_sum_floats(g, ld));
    c.take<float>(chunk_sum_floats(g, ld));
    *bytes = c.bytes();
    return GCN_OK;
}

namespace {
// The aggregation on its own, in a workspace of gcn_aggregate_workspace_bytes that the caller has checked.
int aggregate_in(const gcn_graph *g, const float *in, float *out, int32_t width, int dtype, void *workspace,
                 hipStream_t st) {
    Carver c(workspace);
    const int ld = padded_width(width);
    float *t = c.take<float>((size_t)(g->n + 1) * ld);     // holds float or bfloat16 rows
    float *z = c.take<float>((size_t)(g->n + 1) * ld);
    float *tile_sums = c.take<float>(tile_sum_floats(g, ld));
    float *chunk_sums = c.take<float>(chunk_sum_floats(g, ld));
    const size_t es = dtype == GCN_BF16 ? 2 : 4;
    int rc = pad_rows(in, g->n, width, t, dtype, ld, g->pb.dinv, st);
    if (rc) return rc;
    rc = fill_zero((char *)t + (size_t)g->n * ld * es, (size_t)ld * es, st);
    if (rc) return rc;
    SpmmArgs a = spmm_args(g, t, dtype, ld, z, GCN_F32, ld, ld, width, kEpiNone, tile_sums, chunk_sums);
    rc = spmm_launch(a, st);
    if (rc) return rc;
    return unpad_rows(z, GCN_F32, ld, g->n, width, out, nullptr, st);
}
}  // namespace

int gcn_aggregate(const gcn_graph *g, const float *in, float *out, int32_t width, int dtype, void *workspace,
                  size_t workspace_bytes, void *stream) {
    size_t need = 0;
    int rc = gcn_aggregate_workspace_bytes(g, width, dtype, &need);
    if (rc) return rc;
    if (!in || !out) {
        set_error("gcn_aggregate: null pointer");
        return GCN_EINVAL;
    }
    if (!workspace || !aligned256(workspace) || workspace_bytes < need) {
        set_error("gcn_aggregate: workspace missing, misaligned or smaller than %zu bytes", need);
        return GCN_EWORKSPACE;
    }
    return aggregate_in(g, in, out, width, dtype, workspace, (hipStream_t)stream);
}

// ------------------------------------------------------------------------------------------- gcn_aggregate_static
// Scratch memory of gcn_aggregate_static.  Every GPU the library runs on holds its own copy of this array, at its
// own address, from the moment the code object is loaded there until the process ends.  In host code the array's
// name is only a stand-in for the symbol: the address a kernel may use comes from hipGetSymbolAddress, asked once
// per device with that device current, and is what every launch and copy below is given.
static __device__ __align__(256) unsigned char scratch[GCN_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void **out) {
    int dev = -1;
    GCN_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) {
        set_error("gcn_aggregate_static: device ordinal %d outside 0..%d", dev, kMaxDevices - 1);
        return GCN_EINVAL;
    }
    std::lock_guard<std::mutex> lk(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            set_error("gcn_aggregate_static: hipGetSymbolAddress failed on device %d: %s", dev, hipGetErrorString(e));
            return GCN_EHIP;
        }
        if (!aligned256(p)) {
            set_error("gcn_aggregate_static: the scratch array of device %d is not 256-byte aligned", dev);
            return GCN_EHIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return GCN_OK;
}
}  // namespace

int gcn_aggregate_static(const gcn_graph *g, const float *in, float *out, int32_t width, int dtype, void *stream) {
    size_t need = 0;
    int rc = gcn_aggregate_workspace_bytes(g, width, dtype, &need);
    if (rc) return rc;
    if (!in || !out) {
        set_error("gcn_aggregate_static: null pointer");
        return GCN_EINVAL;
    }
    if (need > (size_t)GCN_STATIC_SCRATCH_BYTES) {
        set_error("gcn_aggregate_static: this graph and width need %zu bytes of scratch memory, the built-in array has %zu; "
                  "use gcn_aggregate with a workspace of the caller's",
                  need, (size_t)GCN_STATIC_SCRATCH_BYTES);
        return GCN_EWORKSPACE;
    }
    if (timing_enabled()) {
        set_error("gcn_aggregate_static: kernel timing is on (it creates events); switch it off first");
        return GCN_EINVAL;
    }
    void *ws = nullptr;
    rc = static_scratch(&ws);
    if (rc) return rc;
    return aggregate_in(g, in, out, width, dtype, ws, (hipStream_t)stream);
}

// ------------------------------------------------------------------------------------------- subgraph approximation
int gcn_augment_workspace_bytes(int64_t n, size_t *bytes) {
    if (!bytes || n <= 0 || n >= 0x7ffffff0) {
        set_error("gcn_augment_workspace_bytes: bad argument");
        return GCN_EINVAL;
    }
    *bytes = augment_workspace_bytes(n);
    return GCN_OK;
}

int gcn_augment_partition(int64_t n, int64_t nnz, const int64_t *rowptr, const int32_t *col, const int32_t *part,
                          int32_t n_parts, int32_t p, double overlap, uint64_t seed, void *workspace,
                          size_t workspace_bytes, int64_t *n_out, int64_t *n_local, int64_t *nnz_out,
                          int32_t *vertices, int64_t *rowptr_out, int32_t *col_out, void *stream) {
    if (!rowptr || (!col && nnz > 0) || !part || !n_out || !n_local || !nnz_out || !vertices || !rowptr_out ||
        (!col_out && nnz > 0) || n <= 0 || n >= 0x7ffffff0 || nnz < 0 || n_parts < 1 || n_parts > 1024 || p < 0 ||
        p >= n_parts || !(overlap >= 0.0)) {
        set_error("gcn_augment_partition: null pointer or bad size (1 <= n_parts <= 1024, 0 <= p < n_parts, overlap >= 0)");
        return GCN_EINVAL;
    }
    size_t need = augment_workspace_bytes(n);
    if (!workspace || !aligned256(workspace) || workspace_bytes < need) {
        set_error("gcn_augment_partition: workspace missing, misaligned or smaller than %zu bytes", need);
        return GCN_EWORKSPACE;
    }
    hipStream_t st = (hipStream_t)stream;
    // the same checks as for any graph: monotone row pointers, columns in range
    int32_t *flags = (int32_t *)workspace;   // first words of the workspace, rewritten by the build below
    int rc = fill_zero(flags, 16 * sizeof(int32_t), st);
    if (rc) return rc;
    rc = prep_validate(n, nnz, rowptr, col, flags, st);
    if (rc) return rc;
    int32_t host_flags[16];
    GCN_HIP(hipMemcpyAsync(host_flags, flags, sizeof(host_flags), hipMemcpyDeviceToHost, st));
    GCN_HIP(hipStreamSynchronize(st));
    if (host_flags[0]) {
        set_error("gcn_augment_partition: invalid CSR (%s)", (host_flags[0] & 1) ? "rowptr" : "column index out of range");
        return GCN_EGRAPH;
    }
    return augment_partition(n, rowptr, col, part, n_parts, p, overlap, seed, workspace, n_out, n_local, nnz_out,
                             vertices, rowptr_out, col_out, st);
}

int gcn_gather_rows(const void *src, size_t row_bytes, const int32_t *idx, int64_t n_idx, void *dst, void *stream) {
    if (!src || !idx || !dst || n_idx < 0) {
        set_error("gcn_gather_rows: null pointer or negative count");
        return GCN_EINVAL;
    }
    return gather_rows(src, row_bytes, idx, n_idx, dst, (hipStream_t)stream);
}

// ------------------------------------------------------------------------------------------- model
int gcn_model_workspace_bytes(const gcn_graph *g, int32_t n_layers, const int32_t *dims, int dtype, size_t *bytes) {
    if (!g || !bytes || (dtype != GCN_F32 && dtype != GCN_BF16) || check_dims(n_layers, dims, dtype)) {
        set_error("gcn_model_workspace_bytes: bad argument");
        return GCN_EINVAL;
    }
    gcn_model m;
    m.g = g;
    m.dtype = dtype;
    m.L = n_layers;
    m.l1_cached = want_l1_cached(n_layers, dims);
    m.l1_split = want_l1_split(dtype, dims[0]);
    for (int l = 0; l < n_layers; ++l)
        m.layers.push_back(Layer{dims[l], dims[l + 1], padded_width(dims[l]), padded_width(dims[l + 1]), nullptr,
                                 nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr});
    Carver c(nullptr);
    carve_model(c, m);
    *bytes = c.bytes();
    return GCN_OK;
}

int gcn_model_create(gcn_model **out, const gcn_graph *g, int32_t n_layers, const int32_t *dims, int dtype,
                     float dropout_p, uint64_t seed, void *workspace, size_t workspace_bytes, void *stream) {
    if (out) *out = nullptr;
    if (!out || !g || check_dims(n_layers, dims, dtype == GCN_BF16 ? GCN_BF16 : GCN_F32)) {
        set_error("gcn_model_create: null pointer or bad layer widths (1..16 layers, input <= 4096 wide, other widths <= 256 "
                  "in float32 and <= 512 in bfloat16)");
        return GCN_EINVAL;
    }
    if ((dtype != GCN_F32 && dtype != GCN_BF16) || dtype != g->store_dtype) {
        set_error("gcn_model_create: dtype must be GCN_F32 or GCN_BF16 and equal to the graph's storage type");
        return GCN_EINVAL;
    }
    if (dims[0] != g->f || dims[n_layers] != g->n_classes) {
        set_error("gcn_model_create: dims[0] must be %d and dims[L] must be %d", g->f, g->n_classes);
        return GCN_EINVAL;
    }
    if (!(dropout_p >= 0.0f && dropout_p < 1.0f)) {
        set_error("gcn_model_create: dropout_p must be in [0, 1)");
        return GCN_EINVAL;
    }
    size_t need = 0;
    int rc = gcn_model_workspace_bytes(g, n_layers, dims, dtype, &need);
    if (rc) return rc;
    if (!workspace || !aligned256(workspace) || workspace_bytes < need) {
        set_error("gcn_model_create: workspace missing, misaligned or smaller than %zu bytes", need);
        return GCN_EWORKSPACE;
    }
    gcn_model *m = new (std::nothrow) gcn_model;
    if (!m) {
        set_error("out of host memory");
        return GCN_EINVAL;
    }
    m->g = g;
    m->L = n_layers;
    m->dtype = dtype;
    m->p = dropout_p;
    m->seed = seed;
    m->l1_cached = want_l1_cached(n_layers, dims);
    m->l1_split = want_l1_split(dtype, dims[0]);
    for (int l = 0; l < n_layers; ++l)
        m->layers.push_back(Layer{dims[l], dims[l + 1], padded_width(dims[l]), padded_width(dims[l + 1]), nullptr,
                                  nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr});
    Carver c(workspace);
    carve_model(c, *m);
    if (c.bytes() != need) {   // the measuring pass and this one must lay out the same buffers
        set_error("gcn_model_create: internal layout mismatch (%zu bytes carved, %zu measured)", c.bytes(), need);
        delete m;
        return GCN_EINVAL;
    }
    // zero everything once: padding columns, the extra zero rows and the weights start at zero
    hipStream_t st = (hipStream_t)stream;
    rc = fill_zero(workspace, need, st);
    if (!rc && m->l1_cached) {
        // P = A_hat X, in column slabs the aggregation kernel can cover with one wave per row
        rc = scale_rows(g->x, m->xs, dtype, g->n, g->ldf, g->pb.dinv, st);
        const int slab = dtype == GCN_BF16 ? 512 : 256;
        const size_t es = dtype == GCN_BF16 ? 2 : 4;
        for (int c0 = 0; !rc && c0 < g->ldf; c0 += slab) {
            const int cols = g->ldf - c0 < slab ? g->ldf - c0 : slab;
            SpmmArgs a = spmm_args(g, (const char *)m->xs + c0 * es, dtype, g->ldf, (char *)m->pax + c0 * es, dtype,
                                   g->ldf, cols, g->f, kEpiNone, m->tile_sums, m->chunk_sums, m->gather_sums);
            rc = spmm_launch(a, st);
        }
    }
    if (!rc && m->l1_split) {
        const float *src = (const float *)(m->l1_cached ? m->pax : g->x);
        rc = pack_rows(src, g->ldf, g->n, g->ldf, m->sp_a, true, st);
        if (!rc && m->sp_at) rc = pack_transposed(src, g->ldf, g->n, g->ldf, m->sp_at, true, st);
    }
    if (rc) {
        delete m;
        return rc;
    }
    *out = m;
    return GCN_OK;
}

int gcn_model_destroy(gcn_model *m) {
    delete m;
    return GCN_OK;
}

int gcn_set_weights(gcn_model *m, const float *flat, int on_host, void *stream) {
    if (!m || !flat) {
        set_error("gcn_set_weights: null pointer");
        return GCN_EINVAL;
    }
    hipStream_t st = (hipStream_t)stream;
    size_t off = 0;
    for (auto &ly : m->layers) {
        const size_t cnt = (size_t)ly.d_in * ly.d_out;
        if (on_host) {
            // stage through the (currently idle) gradient buffer, then spread into the padded layout
            GCN_HIP(hipMemcpyAsync(ly.dw, flat + off, cnt * sizeof(float), hipMemcpyHostToDevice, st));
            GCN_HIP(hipStreamSynchronize(st));
            int rc = pad_rows(ly.dw, ly.d_in, ly.d_out, ly.w, GCN_F32, ly.ld_out, nullptr, st);
            if (rc) return rc;
            GCN_HIP(hipStreamSynchronize(st));
            rc = fill_zero(ly.dw, (size_t)ly.ld_in * ly.ld_out * sizeof(float), st);
            if (rc) return rc;
        } else {
            int rc = pad_rows(flat + off, ly.d_in, ly.d_out, ly.w, GCN_F32, ly.ld_out, nullptr, st);
            if (rc) return rc;
        }
        if (m->dtype == GCN_BF16) {
            int rc = weight_copies(ly.w, ly.ld_in, ly.ld_out, ly.wb, ly.wbt, ly.ld_in, st);
            if (rc) return rc;
        }
        // new weights, fresh optimiser state
        int rc = fill_zero(ly.am, (size_t)ly.ld_in * ly.ld_out * sizeof(float), st);
        if (!rc) rc = fill_zero(ly.av, (size_t)ly.ld_in * ly.ld_out * sizeof(float), st);
        if (rc) return rc;
        off += cnt;
    }
    m->adam_steps = 0;
    m->have_forward = m->have_loss = m->have_backward = false;
    return GCN_OK;
}

int gcn_get_tensor(gcn_model *m, int which, int layer, float *dst, size_t dst_floats, void *stream) {
    if (!m || !dst) {
        set_error("gcn_get_tensor: null pointer");
        return GCN_EINVAL;
    }
    hipStream_t st = (hipStream_t)stream;
    if (which == GCN_T_LOGITS) layer = m->L;
    if (layer < 1 || layer > m->L) {
        set_error("gcn_get_tensor: layer %d out of range", layer);
        return GCN_EINVAL;
    }
    const Layer &ly = m->layers[layer - 1];
    const int64_t n = m->g->n;
    const void *src = nullptr;
    int src_dtype = m->dtype;
    int ld = ly.ld_out, cols = ly.d_out;
    int64_t rows = n;
    const float *rowdiv = nullptr;
    bool ok = true;
    switch (which) {
        case GCN_T_W: src = ly.w; src_dtype = GCN_F32; rows = ly.d_in; break;
        case GCN_T_DW: src = ly.dw; src_dtype = GCN_F32; rows = ly.d_in; ok = m->have_backward; break;
        case GCN_T_H: src = ly.h; ok = m->have_forward && layer < m->L; break;
        case GCN_T_LOGITS: src = ly.h; src_dtype = GCN_F32; ok = m->have_forward; break;
        case GCN_T_G: src = ly.g; ok = m->have_backward && !(layer == 1 && m->l1_cached); break;
        case GCN_T_DZ:
            src = ly.dzs;
            rowdiv = (layer == 1 && m->l1_cached) ? nullptr : m->g->pb.dinv;   // stored without D^-1/2 in that case
            ok = m->have_backward;
            break;
        default: ok = false;
    }
    if (!ok || !src) {
        set_error("gcn_get_tensor: tensor %d of layer %d is not available now", which, layer);
        return GCN_EINVAL;
    }
    if (dst_floats < (size_t)rows * cols) {
        set_error("gcn_get_tensor: destination holds %zu floats, %zu needed", dst_floats, (size_t)rows * cols);
        return GCN_EINVAL;
    }
    return unpad_rows(src, src_dtype, ld, rows, cols, dst, rowdiv, st);
}

namespace {

// c = act(rowscale * (A W_1)) with A = X or P from its packed form; W_1^T is packed first
int l1_split_forward(gcn_model *m, float *c, const float *rowscale, const Activation *act, hipStream_t st,
                     const PlaneSink *sink = nullptr) {
    const Layer &ly = m->layers[0];
    int rc = pack_transposed(ly.w, ly.ld_out, ly.ld_in, ly.ld_out, m->sp_wt, false, st);
    if (rc) return rc;
    return gemm_split(m->sp_a, m->sp_wt, c, ly.ld_out, m->g->n, ly.ld_in, ly.ld_out, rowscale, act, st, sink);
}

// dW_1 = P^T dZ_1 the same way: `rows` = dZ_1 [n x ld_out] is put in the order the product's right operand is read
// in unless its producer left it in m->sp_gu that way; the left operand P^T was packed when the model was made
int l1_split_backward(gcn_model *m, const float *rows, bool have_units, hipStream_t st) {
    const Layer &ly = m->layers[0];
    int rc = have_units ? GCN_OK : units_from_rows(rows, ly.ld_out, m->g->n, ly.ld_out, m->sp_gu, st);
    if (rc) return rc;
    return gemm_split_tn(m->sp_at, m->sp_gu, (int)round_up(ly.ld_out, 32), ly.dw, ly.ld_out, ly.ld_in, m->g->n,
                         ly.ld_out, m->partials, m->partial_floats, st);
}

}  // namespace

int gcn_forward(gcn_model *m, int training, void *stream) {
    if (!m) {
        set_error("gcn_forward: null model");
        return GCN_EINVAL;
    }
    hipStream_t st = (hipStream_t)stream;
    const gcn_graph *g = m->g;
    const bool bf = m->dtype == GCN_BF16;
    const void *h_prev = g->x;
    int ld_prev = g->ldf;
    for (int l = 1; l <= m->L; ++l) {
        Layer &ly = m->layers[l - 1];
        Activation act{l < m->L ? kActRelu : kActNone, ly.d_out, 0u, 1.0f, 0ull};
        if (l < m->L && training && m->p > 0.0f) {
            act.drop_threshold = (uint32_t)std::floor((double)m->p * 4294967296.0);
            act.keep_scale = (float)(1.0 / (1.0 - (double)m->p));
            act.drop_key = host_mix64(host_mix64(m->seed) ^ (m->epoch * 0xD1B54A32D192ED03ull) ^
                                      ((uint64_t)l * 0x8CB92BA72F3D8DD7ull));
        }
        if (l == 1 && m->l1_cached) {
            // H_1 = act(P W_1), P = A_hat X
            const int t_nn = timing_open(kTimeGemmNN, ly.d_out, st);
            int rc = bf ? gemm_bf16_nn(m->pax, g->ldf, ly.wbt, ly.ld_in, ly.h, ly.ld_out, g->n, ly.ld_in, ly.ld_out, nullptr,
                                       &act, st)
                     : m->l1_split
                        ? l1_split_forward(m, (float *)ly.h, nullptr, &act, st)
                        : gemm_nn((const float *)m->pax, g->ldf, ly.w, ly.ld_out, (float *)ly.h, ly.ld_out, g->n, ly.ld_in,
                                  ly.ld_out, nullptr, &act, st);
            timing_close(t_nn, st);
            if (rc) return rc;
            h_prev = ly.h;
            ld_prev = ly.ld_out;
            continue;
        }
        // Z = A_hat-aggregate(T), T = D^-1/2 (H_{l-1} W_l); hidden layers: H = relu(Z) [* keep / (1 - p)]; the logits
        // stay float.  The product also leaves T in the form the aggregation's tile product reads, when it runs one.
        SpmmArgs a = spmm_args(g, ly.t, m->dtype, ly.ld_out, ly.h, l < m->L ? m->dtype : GCN_F32, ly.ld_out, ly.ld_out,
                               ly.d_out, l < m->L ? kEpiRelu : kEpiNone, m->tile_sums, m->chunk_sums, m->gather_sums);
        const PlaneSink sink = tiles_plane_sink(a);
        a.planes_ready = sink.planes != nullptr;
        const int t_nn = timing_open(kTimeGemmNN, ly.d_out, st);
        int rc = bf ? gemm_bf16_nn(h_prev, ld_prev, ly.wbt, ly.ld_in, ly.t, ly.ld_out, g->n, ly.ld_in, ly.ld_out,
                                   g->pb.dinv, nullptr, st)
                 : (l == 1 && m->l1_split)
                    ? l1_split_forward(m, (float *)ly.t, g->pb.dinv, nullptr, st, &sink)
                    : gemm_nn((const float *)h_prev, ld_prev, ly.w, ly.ld_out, (float *)ly.t, ly.ld_out, g->n, ly.ld_in,
                              ly.ld_out, g->pb.dinv, nullptr, st, &sink);
        timing_close(t_nn, st);
        if (rc) return rc;
        a.drop_threshold = act.drop_threshold;
        a.keep_scale = act.keep_scale;
        a.drop_key = act.drop_key;
        rc = spmm_launch(a, st);
        if (rc) return rc;
        h_prev = ly.h;
        ld_prev = ly.ld_out;
    }
    m->have_forward = true;
    m->trained_forward = training && m->p > 0.0f;
    m->have_loss = m->have_backward = false;
    m->dz_units_ready = false;   // (the aggregations above reused the buffer)
    return GCN_OK;
}

int gcn_loss_acc(gcn_model *m, float *loss, float *acc, void *stream) {
    if (!m || !m->have_forward) {
        set_error("gcn_loss_acc: call gcn_forward first");
        return GCN_EINVAL;
    }
    hipStream_t st = (hipStream_t)stream;
    const gcn_graph *g = m->g;
    Layer &ly = m->layers[m->L - 1];
    // dLoss/dlogits is the input of the backward pass's first aggregation: the loss kernel writes it in the tile
    // product's order too, when that aggregation runs one (same arguments as in gcn_backward)
    const SpmmArgs next = spmm_args(g, ly.dzs, m->dtype, ly.ld_out, ly.g, m->dtype, ly.ld_out, ly.ld_out, ly.d_out,
                                    kEpiNone, m->tile_sums, m->chunk_sums, m->gather_sums, true);
    PlaneSink sink = tiles_plane_sink(next);
    if (!loss_can_sink(ly.d_out, m->dtype)) sink.planes = nullptr;
    const int t_loss = timing_open(kTimeLoss, ly.d_out, st);
    int rc = loss_forward(g->n, ly.d_out, (const float *)ly.h, ly.ld_out, g->labels, g->mask, g->pb.dinv, g->n_train,
                          ly.dzs, m->dtype, ly.ld_out, m->loss_part, m->corr_part, m->result, m->result_correct, st,
                          &sink);
    timing_close(t_loss, st);
    if (rc) return rc;
    m->have_loss = true;
    m->dz_units_ready = sink.planes != nullptr;
    if (loss || acc) {
        float host[2];
        GCN_HIP(hipMemcpyAsync(host, m->result, sizeof(host), hipMemcpyDeviceToHost, st));
        GCN_HIP(hipStreamSynchronize(st));
        if (loss) *loss = host[0];
        if (acc) *acc = host[1];
    }
    return GCN_OK;
}

int gcn_loss_acc_counts(gcn_model *m, int64_t *correct, int64_t *n_train, void *stream) {
    if (!m || !m->have_loss) {
        set_error("gcn_loss_acc_counts: call gcn_loss_acc first");
        return GCN_EINVAL;
    }
    hipStream_t st = (hipStream_t)stream;
    long long host = 0;
    GCN_HIP(hipMemcpyAsync(&host, m->result_correct, sizeof(host), hipMemcpyDeviceToHost, st));
    GCN_HIP(hipStreamSynchronize(st));
    if (correct) *correct = (int64_t)host;
    if (n_train) *n_train = m->g->n_train;
    return GCN_OK;
}

int gcn_backward(gcn_model *m, void *stream) {
    if (!m || !m->have_forward || !m->have_loss) {
        set_error("gcn_backward: call gcn_forward and gcn_loss_acc first");
        return GCN_EINVAL;
    }
    hipStream_t st = (hipStream_t)stream;
    const gcn_graph *g = m->g;
    const float keep_scale = m->trained_forward ? (float)(1.0 / (1.0 - (double)m->p)) : 1.0f;
    const bool bf = m->dtype == GCN_BF16;
    // the kernel that wrote this layer's dZ also left it in the tile product's order (the loss kernel for the last
    // layer, the input-gradient product for the others); good for one pass: later aggregations reuse the buffer
    bool planes_ready = m->dz_units_ready;
    m->dz_units_ready = false;
    bool aux_pending = false;    // a weight gradient is running on the graph's stream
    const bool split_tn = m->sp_at != nullptr;   // dW_1 = P^T dZ_1 on the bfloat16 instruction
    bool gu_ready = false;       // its right operand is in m->sp_gu
    for (int l = m->L; l >= 1; --l) {
        Layer &ly = m->layers[l - 1];
        if (l == 1 && m->l1_cached) {
            // dW_1 = P^T dZ_1  (dzs of layer 1 was written without D^-1/2)
            int rc;
            if (aux_pending) {
                GCN_HIP(hipStreamWaitEvent(st, g->ev_aux, 0));
                aux_pending = false;
            }
            const int t_tn = timing_open(kTimeGemmTN, ly.d_out, st);
            if (bf) {
                int splits = 0;
                rc = gemm_bf16_tn_partials(m->pax, g->ldf, ly.dzs, ly.ld_out, ly.ld_out, g->n, ly.ld_in, ly.ld_out,
                                           m->partials, m->partial_floats, &splits, st);
                if (rc) return rc;
                rc = reduce_partials(m->partials, splits, (size_t)ly.ld_in * ly.ld_out, ly.dw, st);
            } else if (split_tn) {
                rc = l1_split_backward(m, (const float *)ly.dzs, gu_ready, st);
            } else {
                rc = gemm_tn((const float *)m->pax, g->ldf, (const float *)ly.dzs, ly.ld_out, ly.dw, ly.ld_out, g->n,
                             ly.ld_in, ly.ld_out, m->partials, m->partial_floats, st);
            }
            timing_close(t_tn, st);
            if (rc) return rc;
            continue;
        }
        // G = A_hat dZ_l  (dzs already carries D^-1/2)
        // (the rows of dZ_L outside the train mask are zero: the loss kernel writes them so)
        SpmmArgs a = spmm_args(g, ly.dzs, m->dtype, ly.ld_out, ly.g, m->dtype, ly.ld_out, ly.ld_out, ly.d_out, kEpiNone,
                               m->tile_sums, m->chunk_sums, m->gather_sums, l == m->L);
        a.planes_ready = planes_ready;
        planes_ready = false;
        int rc = spmm_launch(a, st);
        if (rc) return rc;
        // dW_l = H_{l-1}^T G.  Nothing in the rest of the pass needs it, so above layer 1 it runs on the graph's own
        // stream beside the input gradient of the layer below (knob "tn_beside"); the pass waits for it before the
        // next weight gradient (same buffer of partial matrices) and at its end.
        const void *h_prev = l > 1 ? m->layers[l - 2].h : g->x;
        if (aux_pending) {
            GCN_HIP(hipStreamWaitEvent(st, g->ev_aux, 0));
            aux_pending = false;
        }
        // (only when an aggregation follows below: with layer 1 from the cached A_hat X the pass would just wait for
        // it one product later; measured there 0.563 against 0.554 ms per epoch, here 1.099 against 1.112 ms)
        const bool beside = l > 1 && !(l == 2 && m->l1_cached) && g->side && g->ev_aux && tunable("tn_beside", 1) != 0;
        hipStream_t tn_st = st;
        if (beside) {
            GCN_HIP(hipEventRecord(g->ev_fork, st));
            GCN_HIP(hipStreamWaitEvent(g->side, g->ev_fork, 0));
            tn_st = g->side;
        }
        const int t_tn = timing_open(kTimeGemmTN, ly.d_out, tn_st);
        if (bf) {
            int splits = 0;
            rc = gemm_bf16_tn_partials(h_prev, ly.ld_in, ly.g, ly.ld_out, ly.ld_out, g->n, ly.ld_in, ly.ld_out,
                                       m->partials, m->partial_floats, &splits, tn_st);
            if (!rc) rc = reduce_partials(m->partials, splits, (size_t)ly.ld_in * ly.ld_out, ly.dw, tn_st);
        } else {
            rc = gemm_tn((const float *)h_prev, ly.ld_in, (const float *)ly.g, ly.ld_out, ly.dw, ly.ld_out, g->n,
                         ly.ld_in, ly.ld_out, m->partials, m->partial_floats, tn_st);
        }
        timing_close(t_tn, tn_st);
        if (beside) {   // also after an error: the caller's stream must not run ahead of work already on the other one
            GCN_HIP(hipEventRecord(g->ev_aux, g->side));
            aux_pending = true;
        }
        if (rc) {
            if (aux_pending) GCN_HIP(hipStreamWaitEvent(st, g->ev_aux, 0));
            return rc;
        }
        if (l > 1) {
            // D^-1/2 dZ_{l-1} = D^-1/2 ((G W_l^T) * [H_{l-1} > 0] * keep_scale)
            Layer &lp = m->layers[l - 2];
            const bool aggregated = !(l == 2 && m->l1_cached);
            const float *next_scale = aggregated ? g->pb.dinv : nullptr;
            PlaneSink sink{nullptr, 0, 0};
            if (aggregated) {   // the same arguments as the aggregation of the next round of this loop
                const SpmmArgs next = spmm_args(g, lp.dzs, m->dtype, lp.ld_out, lp.g, m->dtype, lp.ld_out, lp.ld_out,
                                                lp.d_out, kEpiNone, m->tile_sums, m->chunk_sums, m->gather_sums, false);
                sink = tiles_plane_sink(next);
                planes_ready = sink.planes != nullptr;
            } else if (split_tn && tunable("fused_planes", 1) != 0) {   // dZ_1 goes straight into the weight gradient
                sink = PlaneSink{m->sp_gu, (int)((g->n + 31) / 32), (int)round_up(lp.ld_out, 32)};
                gu_ready = true;
            }
            const int t_nt = timing_open(kTimeGemmNT, lp.d_out, st);
            rc = bf ? gemm_bf16_nt(ly.g, ly.ld_out, ly.wb, ly.ld_out, lp.dzs, lp.ld_out, g->n, ly.ld_out, lp.ld_out,
                                   next_scale, lp.h, lp.ld_out, keep_scale, st)
                    : gemm_nt((const float *)ly.g, ly.ld_out, ly.w, ly.ld_out, (float *)lp.dzs, lp.ld_out, g->n,
                              ly.ld_out, lp.ld_out, next_scale, (const float *)lp.h, lp.ld_out, keep_scale, st, &sink);
            timing_close(t_nt, st);
            if (rc) {
                if (aux_pending) GCN_HIP(hipStreamWaitEvent(st, g->ev_aux, 0));
                return rc;
            }
        }
    }
    if (aux_pending) GCN_HIP(hipStreamWaitEvent(st, g->ev_aux, 0));
    m->have_backward = true;
    return GCN_OK;
}

int gcn_sgd_step(gcn_model *m, float lr, void *stream) {
    if (!m || !m->have_backward) {
        set_error("gcn_sgd_step: call gcn_backward first");
        return GCN_EINVAL;
    }
    hipStream_t st = (hipStream_t)stream;
    SgdLayers ls{};
    size_t total = 0;
    for (auto &ly : m->layers) {   // at most kMaxLayers of them: checked when the model was created
        ls.w[ls.n] = ly.w;
        ls.dw[ls.n] = ly.dw;
        total += (size_t)ly.ld_in * ly.ld_out;
        ls.end[ls.n] = total;
        ls.n += 1;
    }
    int rc = sgd_update(ls, lr, st);
    if (rc) return rc;
    if (m->dtype == GCN_BF16)
        for (auto &ly : m->layers) {
            rc = weight_copies(ly.w, ly.ld_in, ly.ld_out, ly.wb, ly.wbt, ly.ld_in, st);
            if (rc) return rc;
        }
    m->epoch += 1;
    m->have_forward = m->have_loss = m->have_backward = false;
    return GCN_OK;
}

int gcn_adam_step(gcn_model *m, float lr, float beta1, float beta2, float eps, void *stream) {
    if (!m || !m->have_backward) {
        set_error("gcn_adam_step: call gcn_backward first");
        return GCN_EINVAL;
    }
    hipStream_t st = (hipStream_t)stream;
    for (auto &ly : m->layers) {
        int rc = adam_update(ly.w, ly.dw, ly.am, ly.av, (size_t)ly.ld_in * ly.ld_out, lr, beta1, beta2, eps,
                             m->adam_steps + 1, st);
        if (rc) return rc;
        if (m->dtype == GCN_BF16) {
            rc = weight_copies(ly.w, ly.ld_in, ly.ld_out, ly.wb, ly.wbt, ly.ld_in, st);
            if (rc) return rc;
        }
    }
    m->adam_steps += 1;
    m->epoch += 1;
    m->have_forward = m->have_loss = m->have_backward = false;
    return GCN_OK;
}

int gcn_average_weights(gcn_model *const *models, int32_t n_models, void *stream) {
    if (!models || n_models < 1 || n_models > 64) {
        set_error("gcn_average_weights: between 1 and 64 models");
        return GCN_EINVAL;
    }
    for (int i = 0; i < n_models; ++i) {
        if (!models[i] || models[i]->L != models[0]->L || models[i]->dtype != models[0]->dtype) {
            set_error("gcn_average_weights: model %d is null or of another shape", i);
            return GCN_EINVAL;
        }
        for (int l = 0; l < models[0]->L; ++l)
            if (models[i]->layers[l].d_in != models[0]->layers[l].d_in ||
                models[i]->layers[l].d_out != models[0]->layers[l].d_out) {
                set_error("gcn_average_weights: model %d has other layer widths", i);
                return GCN_EINVAL;
            }
    }
    hipStream_t st = (hipStream_t)stream;
    for (int l = 0; l < models[0]->L; ++l) {
        float *ws[64];
        for (int i = 0; i < n_models; ++i) ws[i] = models[i]->layers[l].w;
        const Layer &ly = models[0]->layers[l];
        int rc = average_in_place(ws, n_models, (size_t)ly.ld_in * ly.ld_out, st);
        if (rc) return rc;
        for (int i = 0; i < n_models && models[0]->dtype == GCN_BF16; ++i) {
            Layer &li = models[i]->layers[l];
            rc = weight_copies(li.w, li.ld_in, li.ld_out, li.wb, li.wbt, li.ld_in, st);
            if (rc) return rc;
        }
    }
    for (int i = 0; i < n_models; ++i)
        models[i]->have_forward = models[i]->have_loss = models[i]->have_backward = false;
    return GCN_OK;
}

int gcn_adam_update(float *w, const float *dw, float *mom1, float *mom2, size_t count, float lr, float beta1,
                    float beta2, float eps, int64_t step, void *stream) {
    if (!w || !dw || !mom1 || !mom2) {
        set_error("gcn_adam_update: null pointer");
        return GCN_EINVAL;
    }
    return adam_update(w, dw, mom1, mom2, count, lr, beta1, beta2, eps, step, (hipStream_t)stream);
}

// ------------------------------------------------------------------------------------------- timing
int gcn_set_tunable(const char *name, int64_t value) {
    if (!name) {
        set_error("gcn_set_tunable: null name");
        return GCN_EINVAL;
    }
    std::lock_guard<std::mutex> lk(g_knob_mutex);
    for (auto &k : g_knobs)
        if (k.first == name) {
            k.second = value;
            return GCN_OK;
        }
    g_knobs.push_back({std::string(name), value});
    return GCN_OK;
}

int gcn_xcc_ids(int32_t *out, int32_t n_blocks, void *stream) {
    if (!out || n_blocks < 0) {
        set_error("gcn_xcc_ids: null pointer or negative count");
        return GCN_EINVAL;
    }
    return xcc_ids(out, n_blocks, (hipStream_t)stream);
}

int gcn_calibration_copy(const void *src, void *dst, size_t bytes, void *stream) {
    if (!src || !dst) {
        set_error("gcn_calibration_copy: null pointer");
        return GCN_EINVAL;
    }
    return calibration_copy(src, dst, bytes, (hipStream_t)stream);
}

int gcn_timing_enable(int level) {
    std::lock_guard<std::mutex> lk(g_tmutex);
    g_timing = level < 0 ? 0 : (level > 2 ? 2 : level);
    return GCN_OK;
}
int gcn_timing_reset(void) {
    std::lock_guard<std::mutex> lk(g_tmutex);
    for (auto &t : g_launches) g_free_events.push_back({t.start, t.stop});
    g_launches.clear();
    return GCN_OK;
}
int gcn_timing_read(int32_t part, int32_t width, int64_t *launches, double *total_ms) {
    std::lock_guard<std::mutex> lk(g_tmutex);
    int64_t cnt = 0;
    double ms = 0.0;
    for (auto &t : g_launches) {
        if (t.part != part || t.width != width || !t.closed) continue;
        GCN_HIP(hipEventSynchronize(t.stop));
        float one = 0.f;
        GCN_HIP(hipEventElapsedTime(&one, t.start, t.stop));
        ms += one;
        ++cnt;
    }
    if (launches) *launches = cnt;
    if (total_ms) *total_ms = ms;
    return GCN_OK;
}

}  // extern "C"

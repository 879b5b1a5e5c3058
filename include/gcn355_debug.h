/*
 * gcn355_debug.h — measurement aids of libgcn355.so: kernel timing, kernel-variant knobs, calibration and
 * ceiling kernels.  Nothing here is needed to train; benchmarks, profiles and tests use it.
 *
 * Unlike the calls of gcn355.h, the knobs and the timing switch are PROCESS-WIDE state: they are read by
 * gcn_graph_create, gcn_model_create and the launches of every thread.  Set them before creating objects and
 * do not change them while another thread is inside the library.
 */
#ifndef GCN355_DEBUG_H
#define GCN355_DEBUG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ------------------------------------------------------------------------------------------------
 * Kernel timing: when enabled, launches are bracketed by HIP events recorded on the stream the work
 * is launched on (the caller's, or the graph's own for the part of an aggregation that runs there).
 *   level 0  off (default)
 *   level 1  every aggregation as a whole (all its launches and stream hand-overs), and the feature gather of
 *            the GraphSAGE step
 *   level 2  also the parts of an aggregation (gather kernels, operand planes, tile product, join) and the
 *            dense products and the loss; the extra event records put gaps of a few microseconds between
 *            launches, so epoch rates are measured at level 0
 * gcn_timing_read waits for the events and returns, for the closed intervals of (part, width) since the
 * last reset, their count and total milliseconds.  `width`: columns of the aggregated matrix (aggregation
 * parts), columns of the product (dense products), classes (loss), 0 (GraphSAGE gather).
 */
enum gcn_timed_part {
    GCN_TIME_AGGREGATE = 0,   /* a whole aggregation A_hat T                                          */
    GCN_TIME_GATHER = 1,      /* its gather kernels (wave-per-row / phased / lane-group / chunk kernels) */
    GCN_TIME_TILES = 2,       /* the tile product, with the adding-up of cut runs                      */
    GCN_TIME_PLANES = 3,      /* the pass that splits and reorders the input for the tile product      */
    GCN_TIME_JOIN = 4,        /* the launch that adds the two parts and finishes the rows              */
    GCN_TIME_GEMM_NN = 5,     /* H W                                                                   */
    GCN_TIME_GEMM_TN = 6,     /* H^T G with its ordered reduction                                      */
    GCN_TIME_GEMM_NT = 7,     /* G W^T with the ReLU gate                                              */
    GCN_TIME_LOSS = 8,        /* loss, accuracy, dLoss/dlogits                                         */
    GCN_TIME_SAGE_GATHER = 9  /* GraphSAGE: gather and mean of the sampled feature rows                */
};
int gcn_timing_enable(int level);
int gcn_timing_reset(void);
int gcn_timing_read(int32_t part, int32_t width, int64_t *launches, double *total_ms);

/* Benchmark sweeps: sets a named integer knob that selects among equivalent kernel variants or launch
 * shapes.  Results do not depend on any knob beyond rounding order.  Unknown names are stored and ignored.
 *   "cache_ax"          0 / 1 / 2    layer 1 as (A_hat X) W_1 from a cached A_hat X: never / when d_0 <= d_1 (default) /
 *                                    always; read by gcn_model_create
 *   "gemm_split"        0 / 1 / 2    float32 models: layer 1's feature transform on the bfloat16 matrix instruction
 *                                    from three-plane operands: never (the float32 instruction) / when the input is
 *                                    at least 256 wide (default) / always; read by gcn_model_workspace_bytes and
 *                                    gcn_model_create
 *   "gemm_split_tn"     1 / 0        with "gemm_split" and layer 1 from the cached A_hat X: its weight gradient the
 *                                    same way, the vertices (the shared index) cut over workgroups (default) / on
 *                                    the float32 instruction; read by gcn_model_workspace_bytes and gcn_model_create
 *   "split_tn_wgs"      >= 1         workgroups that product aims at when it cuts the shared index (default 256)
 *   "tile_slots"        >= 256       workgroups of the tile product the chip is taken to hold at a time when its
 *                                    work items are planned (default 768); read by gcn_graph_create
 *   "tile_run_min"      >= 8         a row block with up to 1.5 x this many tiles is never cut (default 16)
 *   "spmm_tiles"        -1 / 0 / 1   dense tiles: when they hold a quarter of the entries (default) / never / whenever
 *                                    there is one; read by gcn_graph_create, 0 also per call
 *   "tile_min_entries"  64..4096     entries that make a 128 x 32 tile dense (default 64); read by gcn_graph_create
 *   "tile_chunk"        0 / >= 8     tiles per run when a row block's tiles are cut: three quarters of the average per
 *                                    workgroup place (default) / that many; read by gcn_graph_create
 *   "spmm_overlap"      1 / 0        tile product beside the gather kernel (default) / before it
 *   "spmm_tiles_first"  -1 / 0 / 1   which of the two is launched first, on the caller's stream (the other goes to the
 *                                    graph's own): the gather when it runs the phased schedule, else the tile product
 *                                    (default) / the gather / the tile product
 *   "tile_run_max"      >= 16        tiles per work item of the tile product at most (default 128); read by
 *                                    gcn_graph_create
 *   "fused_planes"      1 / 0        float32 models: the dense product that writes an aggregation's input also writes the
 *                                    tile product's operand planes (default) / a separate pass does
 *   "tn_beside"         1 / 0        backward pass: a layer's weight gradient on the graph's own stream beside the input
 *                                    gradient of the layer below, when an aggregation follows (default) / in line
 *   "spmm_masked"       1 / 0        masked pattern for the last layer's backward aggregation when the train mask
 *                                    holds at most 4/5 of the vertices (default) / never; read by gcn_graph_create
 *   "spmm_phased"       -1 / 0 / 1   phased gather schedule: automatic (default) / never / whenever the shape allows
 *   "phased_balance"    1 / 0        XCD row ranges of the phased schedule by entries (default) / by rows; read by
 *                                    gcn_graph_create
 *   "phased_group"      0 / 1,2,4,8  column ranges (sixteenths of the ids) per phase of the phased schedule: as many as
 *                                    5 MB of input rows allow (default) / that many
 *   "spmm_u"            4 / 8 / 16   gathers in flight per lane group at 17..32 sixteen-byte pieces per row (default 8) */
int gcn_set_tunable(const char *name, int64_t value);

/* Launches n_blocks workgroups of 256 threads and writes, for each, the id of the XCD it ran on
 * (out [dev, n_blocks int32]).  The aggregation kernels assume that workgroup b runs on XCD (b + s) mod 8 for
 * a start s that is the same for all workgroups of a launch. */
int gcn_xcc_ids(int32_t *out, int32_t n_blocks, void *stream);

/* Copies `bytes` (a multiple of 16) from src to dst [dev] with one plain streaming kernel
 * (k_calibration_copy), which reads and writes exactly `bytes` each.  Hardware byte counters collected for
 * the library's kernels are scaled by what they report for this one; its rate is also the streaming
 * ceiling that memory-bound kernels are compared with.  Asynchronous. */
int gcn_calibration_copy(const void *src, void *dst, size_t bytes, void *stream);

/* Ceiling of the gather path.  Every wave adds up `per_wave` rows of `table` [dev, rows x row_floats float32,
 * row_floats a multiple of 4 up to 256] picked by a hash of (wave, step), one 16-byte load per lane, a lane group
 * per row, four loads in flight per lane as in the aggregation kernels, and writes its sum to out [dev, waves x
 * row_floats].  With spread = 0 a wave on XCD x (workgroup id mod 8) picks its rows inside the x-th eighth of the
 * table only, so once each eighth is in its XCD's L2 every gather is an L2 hit: the rate the cache path can
 * deliver to a gather on a matrix of this size.  With spread = 1 rows are picked over the whole table (what a
 * gather without any locality gets).  Bytes gathered = waves x per_wave x row_floats x 4.  Asynchronous. */
int gcn_ceiling_gather(const float *table, int64_t rows, int32_t row_floats, int64_t waves, int32_t per_wave,
                       int spread, float *out, void *stream);

/* Ceiling of the matrix pipes for the instruction the tile product uses: `waves` waves issue `per_wave` times
 * four independent v_mfma_f32_32x32x16_bf16 (32,768 flop each) on registers and store one accumulator to out
 * [dev, waves x 64 float32].  Asynchronous. */
int gcn_ceiling_mfma_bf16(int64_t waves, int32_t per_wave, float *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* GCN355_DEBUG_H */

/*
 * gcn355 — full-batch Kipf-Welling GCN training step on one partition subgraph, for MI355X (gfx950).
 *
 * The unit of work is what one worker of the paper's data-parallel scheme does in one epoch
 * (Section 3.2): it holds a complete copy of the network and trains it, full batch, on its own
 * partition, which has already been extended by a few percent of vertices that approximate the
 * other partitions (Section 3.1, Algorithm 1).  To this library those extra vertices are ordinary
 * rows of the same adjacency and feature matrix; they are simply outside the train mask.
 *
 * Model (Section 4.1): H^l = sigma(A_hat H^{l-1} W^l), H^0 = X, with X holding one feature row
 * per vertex and A the adjacency matrix (Section 2.1).  A_hat, the "normalized adjacency matrix"
 * of the footnote to Section 4.1, is D^-1/2 (A + I) D^-1/2, D = row sums of A + I, A binary.
 * sigma is ReLU on hidden layers; the last layer's output are the logits.  The loss is the
 * softmax cross-entropy averaged over the vertices of the train mask; accuracy (the micro-F1 of
 * Section 2.2, which equals plain accuracy for one label per vertex) is measured on the same mask.
 * No bias terms.  The update is plain SGD.
 *
 * Conventions for every call
 *   - Pointers marked [dev] are device pointers valid on the current HIP device; [host] are host
 *     pointers.  `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - The library allocates no device memory: the caller hands over workspaces (sized by the
 *     *_workspace_bytes calls, 256-byte aligned) and keeps them alive until the matching destroy.
 *     Everything else passed to a create call is copied and may be released once it returns.
 *   - Dense matrices crossing this boundary are row-major, float32, without padding.
 *   - "Tunable" below means a named knob of gcn_set_tunable, declared with the other measurement aids (kernel
 *     timing, calibration and ceiling kernels) in gcn355_debug.h; every default is the measured best.
 *   - Return value: GCN_OK (0) or a negative gcn_status.  No call aborts or throws; after a
 *     failure gcn_last_error() returns a thread-local description.  A failed create leaves *out
 *     NULL.  Calls on one model must not overlap in time (one stream at a time).
 */
#ifndef GCN355_H
#define GCN355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gcn_graph gcn_graph;
typedef struct gcn_model gcn_model;

enum gcn_status {
    GCN_OK = 0,
    GCN_EINVAL = -1,     /* null pointer, bad size, call out of order, empty train mask        */
    GCN_EGRAPH = -2,     /* rowptr not monotone / wrong ends, column out of range, not symmetric */
    GCN_ELABEL = -3,     /* a label outside [0, n_classes)                                     */
    GCN_EWORKSPACE = -4, /* workspace missing, misaligned or too small                         */
    GCN_EHIP = -5        /* a HIP runtime call failed (text in gcn_last_error)                  */
};

/* Storage type of features and activations.  Weights, gradients of weights, the loss and every
 * accumulator are float32 in both modes. */
enum gcn_dtype { GCN_F32 = 0, GCN_BF16 = 1 };

/* Tensors readable with gcn_get_tensor; `layer` counts from 1. */
enum gcn_tensor {
    GCN_T_W = 0,      /* W^l                      d_{l-1} x d_l                                  */
    GCN_T_DW = 1,     /* dLoss/dW^l               d_{l-1} x d_l   (after gcn_backward)           */
    GCN_T_H = 2,      /* H^l, l < L               n x d_l         (after gcn_forward)            */
    GCN_T_LOGITS = 3, /* A_hat H^{L-1} W^L        n x d_L         (layer argument ignored)       */
    GCN_T_G = 4,      /* A_hat (dLoss/dZ^l)       n x d_l         (after gcn_backward)           */
    GCN_T_DZ = 5      /* dLoss/dZ^l, Z^l = A_hat H^{l-1} W^l      n x d_l (after gcn_backward)   */
};

const char *gcn_last_error(void);

/* ------------------------------------------------------------------------------------------------
 * Graph: the partition's adjacency, features, labels and train mask (inputs of Section 2.1/2.2).
 *
 * gcn_graph_create takes the raw adjacency A in CSR form: rowptr [dev, n+1, int64, rowptr[0] = 0,
 * rowptr[n] = nnz_in], col [dev, nnz_in, int32].  Column order inside a row is free, repeated
 * entries and explicit self-loops are allowed; the pattern must be symmetric.  On the GPU it builds
 * the canonical pattern of A + I (columns ascending, distinct, exactly one self-loop per row), the
 * integer degrees d_i = row length, d_i^-1/2, and the row schedule of the aggregation kernels.
 * feat [dev, n x f float32], labels [dev, n, int32 in [0, n_classes)], train_mask [dev, n, uint8,
 * non-zero = in the mask].  store_dtype selects how the library keeps its own copy of X.
 * The call is synchronous (it reads back sizes and error flags).  Errors: GCN_EGRAPH, GCN_ELABEL,
 * GCN_EINVAL (empty mask, n <= 0 ...), GCN_EWORKSPACE.
 */
int gcn_graph_workspace_bytes(int64_t n, int64_t nnz_in, int32_t f, int store_dtype, size_t *bytes);
int gcn_graph_create(gcn_graph **out, int64_t n, int64_t nnz_in, const int64_t *rowptr, const int32_t *col,
                     const float *feat, int32_t f, int store_dtype, const int32_t *labels,
                     const uint8_t *train_mask, int32_t n_classes, void *workspace, size_t workspace_bytes,
                     void *stream);
int gcn_graph_destroy(gcn_graph *g);

/* Sizes: n, E = nonzeros of A + I, size of the train mask, largest degree.  Any pointer may be NULL. */
int gcn_graph_info(const gcn_graph *g, int64_t *n, int64_t *nnz, int64_t *n_train, int32_t *max_degree);

/* Dense tiles.  The aggregation of Section 4.1's layer rule (the nnz(A) F term of Section 5.4's cost model)
 * runs in two parts when the adjacency pattern has dense blocks, as the partitions of a community-structured
 * graph do (Section 3) and as the rows and columns of the vertices that stand in for the other partitions do
 * (Section 3.1): the pattern is cut into aligned tiles of 128 rows x 32 columns; tiles with at least
 * `tile_min_entries` stored entries (tunable, default 64, allowed 64..4096) are kept as 128 words of 32 bits and
 * multiplied on the matrix cores, all other entries stay in a residual CSR that is gathered as usual.  The
 * split is used when the dense tiles hold at least a quarter of the entries (tunable "spmm_tiles": -1 this rule,
 * 0 never, 1 whenever there is a dense tile; read at gcn_graph_create, and 0 also switches the form off per
 * call), for matrices of at most 256 columns in either storage type.
 * Arithmetic of the tile product: a float32 value is split exactly into three bfloat16 numbers (8 + 8 + 8
 * significant bits), ones and zeros are exact too, and three passes of the bfloat16 matrix instruction add the
 * products into float32 accumulators: the same terms as the gather form adds, in float32, in another order
 * (values below 2^-110 in magnitude lose their last bits).  bfloat16 rows take one pass.  A non-finite value in
 * a row of the aggregated matrix reaches, through 0 x inf, all 128 rows of the tiles that cover it.
 * Streams: with the split in use the tile product (a pass that splits and reorders the input, then the product)
 * runs beside the gather kernel, one of the two on the caller's stream and the other on a stream of default
 * priority that the graph owns (the gather on the caller's where it runs the phased schedule, else the tile product);
 * fork and join are done with events, so the caller's stream order is kept, and a last launch adds the two
 * parts.  Tunable "spmm_overlap": 1 = this (default), 0 = one launch after the other on the caller's stream
 * (float32 storage; bfloat16 matrices are then gathered whole).  Because that stream and its events belong to the graph, calls that aggregate over one graph
 * (gcn_aggregate, gcn_model_create, gcn_forward, gcn_backward) must not overlap in time, whatever streams they
 * are given.
 * gcn_graph_tile_info: number of dense tiles, stored entries inside them, 1 if the split is in use.
 * gcn_graph_get_tiles (only when in use; any pointer may be NULL; asynchronous on `stream` except *res_nnz):
 *   tile_ptr [dev, ceil(n/128)+1 int64] dense tiles of row block i (rows 128 i ..) are tile_ptr[i] .. tile_ptr[i+1]
 *   tile_col [dev, n_tiles int32]       their column tiles (32 columns each), ascending inside a row block
 *   bits     [dev, n_tiles*128 uint32]  word r of tile k: bit c set = entry (128 i + r, 32 tile_col[k] + c)
 *   res_rowptr [dev, n+1 int64], res_col [dev, *res_nnz int32]  the residual pattern, rows sorted
 *   res_nnz  [host] E minus the entries inside dense tiles */
int gcn_graph_tile_info(const gcn_graph *g, int64_t *n_tiles, int64_t *nnz_dense, int32_t *in_use);
int gcn_graph_get_tiles(const gcn_graph *g, int64_t *tile_ptr, int32_t *tile_col, uint32_t *bits,
                        int64_t *res_rowptr, int32_t *res_col, int64_t *res_nnz, void *stream);

/* The masked pattern.  In the backward pass of the last layer the aggregated matrix is dLoss/dlogits of Section 2.2's
 * loss, whose rows are zero for every vertex outside the train mask, so that aggregation runs over the pattern it
 * would gather over anyway (the residual one when dense tiles are in use, else A + I) without the columns of
 * those vertices.  Built by gcn_graph_create when the train mask holds at most four fifths of the vertices
 * (tunable "spmm_masked": 1 this rule (default), 0 never; read at gcn_graph_create); the sums do not change, only
 * zero terms are left out.
 * gcn_graph_get_masked_pattern (an error when the graph has none; rowptr [dev, n+1 int64] and col [dev, int32,
 * room for *nnz entries; ask for *nnz first] may be NULL; asynchronous on `stream` except *nnz [host]). */
int gcn_graph_get_masked_pattern(const gcn_graph *g, int64_t *rowptr, int32_t *col, int64_t *nnz, void *stream);

/* Copies the canonical arrays to caller buffers [dev]: rowptr (n+1 int64), col (E int32), deg (n int32),
 * dinv (n float32).  Any pointer may be NULL.  Asynchronous on `stream`. */
int gcn_graph_get_csr(const gcn_graph *g, int64_t *rowptr, int32_t *col, int32_t *deg, float *dinv, void *stream);

/* out = A_hat in, for a caller matrix [dev, n x width float32] (the aggregation of Section 4.1's layer
 * rule on its own; cost term nnz(A) F of Section 5.4).  `workspace` [dev] of at least
 * gcn_aggregate_workspace_bytes.  Asynchronous. */
int gcn_aggregate_workspace_bytes(const gcn_graph *g, int32_t width, int dtype, size_t *bytes);
int gcn_aggregate(const gcn_graph *g, const float *in, float *out, int32_t width, int dtype, void *workspace,
                  size_t workspace_bytes, void *stream);

/* gcn_aggregate for callers that cannot allocate device memory or size a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments and same result as gcn_aggregate (it runs
 * the same kernels), but the scratch memory (the padded and scaled copy of `in`, the padded result, the tile
 * product's sums and the chunk sums of split rows) is an array of GCN_STATIC_SCRATCH_BYTES bytes built into the
 * library, one copy per GPU, held from the time the library is loaded on that GPU until the process ends.
 * The call allocates nothing on the device (no hipMalloc, no hipFree, no event or stream is created).
 *   - GCN_EWORKSPACE when gcn_aggregate_workspace_bytes(g, width, dtype) exceeds GCN_STATIC_SCRATCH_BYTES (about
 *     (3 n + 2) x width rounded up to 16, x 4 bytes: e.g. 10,000 vertices at width 256, 57,000 at width 41);
 *     use gcn_aggregate then.  GCN_EINVAL while kernel timing is enabled (timing creates events).
 *   - All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU race, whatever
 *     streams and graphs they use.  Calls in stream order are fine; nothing is kept between calls.
 * Asynchronous on `stream`. */
#define GCN_STATIC_SCRATCH_BYTES (32u << 20)
int gcn_aggregate_static(const gcn_graph *g, const float *in, float *out, int32_t width, int dtype, void *stream);

/* ------------------------------------------------------------------------------------------------
 * Subgraph approximation: builds, on the GPU, the input the training step above runs on.
 *
 * gcn_augment_partition computes P_o[p] of Algorithm 1 (breadth-first random sampling, Section 3.1) for
 * partition p of a graph whose vertices carry partition ids part[v] in [0, n_parts), and the subgraph it
 * induces (Section 4: every edge between subgraphs that the sampling did not bring in is dropped).
 *   nts = floor(overlap * N_p / (n_parts - 1)) vertices are wanted from each other partition op.
 *   Level 1 of op = its vertices adjacent to p; level k + 1 = its vertices adjacent to level k and not seen
 *   before.  Levels are taken whole while they fit; from the first that does not, exactly the missing
 *   number is drawn; an empty level ends the search for op.
 *   The paper names no random generator.  The draw keeps the vertices with the smallest
 *   key(v) = mix(mix(seed) ^ v), mix = the SplitMix64 output function (a bijection: no ties).
 * Inputs [dev]: rowptr (n + 1), col (nnz), part (n).  Outputs: *n_out, *n_local, *nnz_out [host];
 * vertices [dev, capacity n]: old ids in new-id order — partition p ascending, then the sampled vertices
 * ascending; rowptr_out [dev, capacity n + 1] and col_out [dev, capacity nnz]: raw CSR of the induced
 * subgraph in new ids, entries of a row in the order of the input row (feed it to gcn_graph_create).
 * Synchronous.  Errors: GCN_EGRAPH (bad CSR), GCN_EINVAL (partition id out of range ...), GCN_EWORKSPACE.
 */
int gcn_augment_workspace_bytes(int64_t n, size_t *bytes);
int gcn_augment_partition(int64_t n, int64_t nnz, const int64_t *rowptr, const int32_t *col, const int32_t *part,
                          int32_t n_parts, int32_t p, double overlap, uint64_t seed, void *workspace,
                          size_t workspace_bytes, int64_t *n_out, int64_t *n_local, int64_t *nnz_out,
                          int32_t *vertices, int64_t *rowptr_out, int32_t *col_out, void *stream);

/* dst[i, :] = src[idx[i], :] for rows of row_bytes bytes (a multiple of 4): features, labels or masks of the
 * vertices gcn_augment_partition lists.  All pointers [dev].  Asynchronous. */
int gcn_gather_rows(const void *src, size_t row_bytes, const int32_t *idx, int64_t n_idx, void *dst, void *stream);

/* ------------------------------------------------------------------------------------------------
 * Model: L layers (1..16) of widths dims[0..L] (dims[0] = f <= 4096, dims[L] = n_classes; dims[1..L] at most 256
 * with GCN_F32 and 512 with GCN_BF16, else GCN_EINVAL), one local copy of the
 * network as each worker holds it (Section 3.2).  dropout_p in [0, 1) applies to hidden activations
 * in training mode only; the keep mask is the integer function
 *     keep(e) = [ (mix(key + e * 0x9E3779B97F4A7C15) >> 32) >= floor(p * 2^32) ],
 *     key = mix(mix(seed) ^ epoch * 0xD1B54A32D192ED03 ^ layer * 0x8CB92BA72F3D8DD7),
 * mix = the SplitMix64 output function, e = row * d_l + column, epoch = number of gcn_sgd_step
 * calls so far.  Weights start at zero; set them with gcn_set_weights.
 *
 * dtype must equal the graph's store_dtype.  With GCN_BF16, X, the hidden activations and the
 * gradients flowing between kernels are stored as bfloat16 (round to nearest even); products run on
 * bfloat16 matrix-core instructions with float32 accumulation; weights (master copy), weight
 * gradients, logits, loss and every sum are float32.
 *
 * Order of the two products per layer (the result is the same, A_hat (H W) = (A_hat H) W): every layer
 * is evaluated as A_hat (H W), except that layer 1 may be evaluated as (A_hat X) W_1 with P = A_hat X
 * computed once in gcn_model_create, because X never changes: then neither the forward nor the backward
 * pass of layer 1 needs an aggregation (dW_1 = P^T dZ_1).  The knob "cache_ax" (gcn_set_tunable, read by
 * gcn_model_workspace_bytes and gcn_model_create) selects: 0 never, 1 (default) when dims[0] <= dims[1],
 * 2 always; it needs n_layers >= 2 and costs two extra copies of X in the workspace.  In that mode
 * GCN_T_G of layer 1 does not exist (gcn_get_tensor returns GCN_EINVAL for it).
 */
int gcn_model_workspace_bytes(const gcn_graph *g, int32_t n_layers, const int32_t *dims, int dtype, size_t *bytes);
int gcn_model_create(gcn_model **out, const gcn_graph *g, int32_t n_layers, const int32_t *dims, int dtype,
                     float dropout_p, uint64_t seed, void *workspace, size_t workspace_bytes, void *stream);
int gcn_model_destroy(gcn_model *m);

/* flat = W^1 | W^2 | ... each d_{l-1} x d_l row-major float32; [host] if on_host else [dev].  Synchronous
 * when on_host. */
int gcn_set_weights(gcn_model *m, const float *flat, int on_host, void *stream);

/* Copies one tensor, unpadded row-major float32, into dst [dev, dst_floats >= rows*cols].  Asynchronous. */
int gcn_get_tensor(gcn_model *m, int which, int layer, float *dst, size_t dst_floats, void *stream);

/* Forward pass of Section 4.1's rule over all layers: for l = 1..L, Z^l = A_hat (H^{l-1} W^l),
 * H^l = relu(Z^l) (times the dropout mask / (1-p) if training != 0 and p > 0).  Asynchronous. */
int gcn_forward(gcn_model *m, int training, void *stream);

/* Masked softmax cross-entropy (mean over the train mask) and accuracy (fraction of masked vertices
 * whose arg-max logit, lowest index on ties, equals the label — the micro-F1 of Section 2.2).  Also
 * stages dLoss/dlogits for gcn_backward.  Needs gcn_forward first.  If loss and acc [host] are both
 * NULL the call only enqueues work; otherwise it waits for the stream and writes them. */
int gcn_loss_acc(gcn_model *m, float *loss, float *acc, void *stream);

/* The integers behind the accuracy of the last gcn_loss_acc: how many masked vertices were classified
 * correctly, and the size of the mask.  Waits for the stream.  Either pointer [host] may be NULL. */
int gcn_loss_acc_counts(gcn_model *m, int64_t *correct, int64_t *n_train, void *stream);

/* Backward pass: for l = L..1, G = A_hat dZ^l (A_hat is symmetric, so the same pattern serves),
 * dW^l = H^{l-1}^T G, dZ^{l-1} = (G W^l^T) * [Z^{l-1} > 0] (* dropout mask / (1-p)).  Needs gcn_forward and
 * gcn_loss_acc first (GCN_EINVAL otherwise).  Asynchronous. */
int gcn_backward(gcn_model *m, void *stream);

/* W^l <- W^l - lr dW^l for all layers; advances the epoch counter.  Needs gcn_backward.  Asynchronous. */
int gcn_sgd_step(gcn_model *m, float lr, void *stream);

/* Adam step for all layers, the optimiser the paper trains KW-GCN with (Section 4.1: Adam, learning rate
 * 0.02; it prints no other constant, the usual ones are beta1 = 0.9, beta2 = 0.999, eps = 1e-8):
 *   m <- beta1 m + (1 - beta1) g,  v <- beta2 v + (1 - beta2) g^2,
 *   W <- W - lr (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps),   t = Adam steps so far + 1.
 * The moments live in the model's workspace and are reset by gcn_set_weights.  Needs gcn_backward;
 * advances the epoch counter like gcn_sgd_step.  Asynchronous. */
int gcn_adam_step(gcn_model *m, float lr, float beta1, float beta2, float eps, void *stream);

/* Parameter aggregation of Section 3.2: at the end of an epoch every worker's weights W_i are replaced by
 * their average W_agg = (1 / n) sum_i W_i (summed in list order).  Here the n models (at most 64, same layer
 * widths and storage type, typically one per partition) live on one GPU; across GPUs the same step is one
 * all-reduce of the flat weight buffer.  Optimiser moments are left alone: the paper averages parameters.
 * All models' work must be on, or ordered before, `stream`.  Asynchronous. */
int gcn_average_weights(gcn_model *const *models, int32_t n_models, void *stream);

/* The same update on caller buffers [dev, count floats each]: w, the gradient dw, and the two moment
 * arrays; `step` is t above (>= 1).  Asynchronous. */
int gcn_adam_update(float *w, const float *dw, float *mom1, float *mom2, size_t count, float lr, float beta1,
                    float beta2, float eps, int64_t step, void *stream);

/* ------------------------------------------------------------------------------------------------------------
 * GraphSAGE with the element-wise mean as propagation rule, two layers, trained in batches (Section 4.1: sample a
 * fixed number of neighbours, aggregate their features, predict; batch size 256, Adam).  Per batch of B target
 * vertices, with N(v) = the row of v in the graph without v itself:
 *   level-1 instances  m = i (1 + S2) + t:  t = 0 the target batch[i] itself, t = 1..S2 its sampled neighbours
 *   h_m  = relu(W1^T [x_u | (1 / S1) sum of the S1 sampled rows of X])          u = the vertex of instance m
 *   z_i  = W2^T [h_(i,0) | (1 / S2) sum over t = 1..S2 of h_(i,t)]              logits of target i
 *   loss = softmax cross-entropy averaged over the batch (labels of the graph), Section 2.2
 * Where the paper is silent: own row and mean are concatenated; no normalisation of embeddings; neighbours are
 * drawn uniformly with replacement (always S draws; a vertex without neighbours contributes zeros); instances are
 * not deduplicated; draw j of instance m at level l (1 = outer, S1; 2 = the targets' own, S2) is neighbour number
 * floor(u d) of the d sorted neighbours, u = top 32 bits of mix(key_l + (m S + j) g) / 2^32, g = 0x9E3779B97F4A7C15,
 * mix(z) = the SplitMix64 output function of z + g, key_l = mix(mix(seed) ^ step * 0xD1B54A32D192ED03 ^
 * l * 0x8CB92BA72F3D8DD7).  The graph must store float32 features (GCN_F32); at most 256 hidden units and classes.
 * Weights, caller layout: w1 [2 f x hidden] row-major (rows 0..f-1 multiply the vertex's own features, rows
 * f..2f-1 the mean), w2 [2 hidden x classes] likewise.  All device pointers; calls are asynchronous on `stream`
 * except where noted.  The workspace (gcn_sage_workspace_bytes, 256-byte aligned) belongs to the object until
 * gcn_sage_destroy; the graph must outlive it.  Errors: GCN_EINVAL, GCN_EWORKSPACE, GCN_EHIP. */
typedef struct gcn_sage gcn_sage;
int gcn_sage_workspace_bytes(const gcn_graph *g, int32_t hidden, int32_t s1, int32_t s2, int32_t max_batch,
                             size_t *bytes);
int gcn_sage_create(gcn_sage **out, const gcn_graph *g, int32_t hidden, int32_t s1, int32_t s2, int32_t max_batch,
                    uint64_t seed, void *workspace, size_t workspace_bytes, void *stream);
int gcn_sage_destroy(gcn_sage *s);
/* Also clears the Adam moments and the step count. */
int gcn_sage_set_weights(gcn_sage *s, const float *w1, const float *w2, void *stream);
/* Samples (key from the object's seed and `step`), both layers.  batch [dev, n_batch int32, 1 <= n_batch <=
 * max_batch, entries in [0, n), repeats allowed] is copied.  Asynchronous, so an entry outside [0, n) cannot be
 * refused here: it is computed as a vertex without features and neighbours, with label 0, and raises a flag that
 * the next gcn_sage_loss_acc with a host pointer reports as GCN_EINVAL (and clears). */
int gcn_sage_forward(gcn_sage *s, const int32_t *batch, int32_t n_batch, uint64_t step, void *stream);
/* Loss, accuracy = correct / n_batch, number of correct arg-max predictions (ties: lowest class) of the last
 * forward; also leaves dLoss/dlogits for gcn_sage_backward.  loss, acc, correct [host] may be NULL; if all are,
 * the call is asynchronous. */
int gcn_sage_loss_acc(gcn_sage *s, float *loss, float *acc, int64_t *correct, void *stream);
int gcn_sage_backward(gcn_sage *s, void *stream);
/* Adam (Kingma & Ba) on both weight matrices, bias-corrected, step count kept by the object. */
int gcn_sage_adam_step(gcn_sage *s, float lr, float beta1, float beta2, float eps, void *stream);
enum {
    GCN_SAGE_W1 = 0,       /* float [2 f x hidden]                                              */
    GCN_SAGE_W2 = 1,       /* float [2 hidden x classes]                                        */
    GCN_SAGE_DW1 = 2,      /* float [2 f x hidden]            after gcn_sage_backward           */
    GCN_SAGE_DW2 = 3,      /* float [2 hidden x classes]      after gcn_sage_backward           */
    GCN_SAGE_H1 = 4,       /* float [n_batch (1 + S2) x hidden]   layer-1 outputs, instance order */
    GCN_SAGE_LOGITS = 5,   /* float [n_batch x classes]                                          */
    GCN_SAGE_C1_MEAN = 6,  /* float [n_batch (1 + S2) x f]    the mean of the sampled feature rows */
    GCN_SAGE_INNER = 7,    /* int32 [n_batch x S2]            sampled neighbours of the targets, -1 = none */
    GCN_SAGE_OUTER = 8     /* int32 [n_batch (1 + S2) x S1]   sampled neighbours of the instances */
};
/* Copies one of the above (of the last batch) to dst [dev, dst_elems elements of its type]. */
int gcn_sage_get_tensor(gcn_sage *s, int which, void *dst, size_t dst_elems, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* GCN355_H */

// GraphSAGE with the element-wise mean as propagation rule, two layers, trained in batches (Section 4.1): the
// second network the method is evaluated on.  One batch step:
//   sample    S2 neighbours for every target, S1 for every level-1 vertex (targets and their samples)
//   layer 1   h_u = relu(W1^T [x_u | mean of the sampled x])     k_sage_concat1 (gather, HBM-bound) + k_gemm<kNN>
//   layer 2   z_v = W2^T [h_v | mean of the sampled h]           k_sage_concat2 + k_gemm<kNN>
//   loss      softmax cross-entropy over the batch                k_loss
//   backward  dW2 = C2^T dZ2, dC2 = dZ2 W2^T, through the mean and the ReLU, dW1 = C1^T dZ1
//   update    Adam
// Level-1 vertices are not deduplicated: every (target, sample) pair is its own instance with its own outer
// samples, so all shapes are fixed by the batch size: C1 is [B (1 + S2)] x 2 f, C2 is B x 2 hidden.
// A neighbour is drawn uniformly with replacement from the row of the vertex without the vertex itself, by a
// counter-based generator: draw j of instance m at a level takes the top 32 bits of mix64(key + (m S + j) golden)
// as a fraction of the neighbour count.  A vertex without neighbours (or a missing vertex, -1) contributes zeros.
#include <new>

#include "common.hpp"
#include "epilogue.hpp"
#include "graph_object.hpp"

using namespace gcn;

namespace {

constexpr int kThreads = 256;
constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;

inline unsigned blocks_for(int64_t items, int per_block) { return (unsigned)((items + per_block - 1) / per_block); }

uint64_t host_mix(uint64_t z) {
    z += kGolden;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
uint64_t level_key(uint64_t seed, uint64_t step, uint64_t level) {
    return host_mix(host_mix(seed) ^ (step * 0xD1B54A32D192ED03ull) ^ (level * 0x8CB92BA72F3D8DD7ull));
}

// One thread per (instance m, draw j): out[m S + j] = a neighbour of nodes[m], or -1.
__global__ void k_sage_sample(const int64_t *__restrict__ rowptr, const int32_t *__restrict__ col,
                              const int32_t *__restrict__ nodes, int64_t n_nodes, int S, uint64_t key,
                              int32_t *__restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_nodes * S) return;
    const int64_t m = i / S;
    const int v = nodes[m];
    int pick = -1;
    if (v >= 0) {
        const int64_t beg = rowptr[v], end = rowptr[v + 1];
        // position of v itself in its sorted row (the canonical pattern holds the diagonal)
        int64_t lo = beg, hi = end;
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            if (col[mid] < v) lo = mid + 1; else hi = mid;
        }
        const bool has_self = lo < end && col[lo] == v;
        const int64_t d = (end - beg) - (has_self ? 1 : 0);
        if (d > 0) {
            const uint64_t r = mix64(key + (uint64_t)i * kGolden);
            int64_t u = (int64_t)(((r >> 32) * (uint64_t)d) >> 32);
            if (has_self && beg + u >= lo) ++u;      // step over the diagonal entry
            pick = col[beg + u];
        }
    }
    out[i] = pick;
}

// nodes1[i (1 + S2)] = batch[i], nodes1[i (1 + S2) + t] = inner[i S2 + t - 1]; labels_b[i] = labels[batch[i]]
__global__ void k_sage_nodes1(const int32_t *__restrict__ batch, const int32_t *__restrict__ inner, int B, int S2,
                              const int32_t *__restrict__ labels, int32_t *__restrict__ nodes1,
                              int32_t *__restrict__ labels_b) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B * (1 + S2)) return;
    const int b = i / (1 + S2), t = i % (1 + S2);
    const int v = batch[b];       // already -1 if it was out of range
    nodes1[i] = t == 0 ? v : inner[b * S2 + t - 1];
    if (t == 0) labels_b[b] = v >= 0 ? labels[v] : 0;
}

// One thread per (instance m, four columns): c1[m] = [x_node | (1 / S1) sum over the S1 sampled rows], the sum in
// ascending draw order.  Bound by the reads of (1 + S1) feature rows per instance.
__global__ __launch_bounds__(kThreads) void k_sage_concat1(const float *__restrict__ x, int ldf,
                                                           const int32_t *__restrict__ nodes1,
                                                           const int32_t *__restrict__ outer, int S1, int64_t n1,
                                                           float *__restrict__ c1) {
    const int quads = ldf / 4;
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n1 * quads) return;
    const int64_t m = i / quads;
    const int c = (int)(i % quads) * 4;
    const int v = nodes1[m];
    float4 self = make_float4(0.f, 0.f, 0.f, 0.f);
    if (v >= 0) self = *reinterpret_cast<const float4 *>(x + (int64_t)v * ldf + c);
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    const int32_t *ids = outer + m * S1;
    int j = 0;
    for (; j + 4 <= S1; j += 4) {      // four rows in flight, added in draw order
        float4 q[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int id = ids[j + u];
            q[u] = id >= 0 ? *reinterpret_cast<const float4 *>(x + (int64_t)id * ldf + c) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            s.x += q[u].x;
            s.y += q[u].y;
            s.z += q[u].z;
            s.w += q[u].w;
        }
    }
    for (; j < S1; ++j) {
        const int id = ids[j];
        if (id >= 0) {
            const float4 q = *reinterpret_cast<const float4 *>(x + (int64_t)id * ldf + c);
            s.x += q.x;
            s.y += q.y;
            s.z += q.z;
            s.w += q.w;
        }
    }
    const float inv = 1.0f / (float)S1;
    float *o = c1 + m * (2 * (int64_t)ldf);
    *reinterpret_cast<float4 *>(o + c) = self;
    *reinterpret_cast<float4 *>(o + ldf + c) = make_float4(s.x * inv, s.y * inv, s.z * inv, s.w * inv);
}

// c2[i] = [h1 of instance 0 of target i | (1 / S2) sum of h1 over its instances 1..S2]
__global__ void k_sage_concat2(const float *__restrict__ h1, int ldh, int B, int S2, float *__restrict__ c2) {
    const int quads = ldh / 4;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B * quads) return;
    const int b = i / quads, c = (i % quads) * 4;
    const float *base = h1 + (int64_t)b * (1 + S2) * ldh + c;
    const float4 self = *reinterpret_cast<const float4 *>(base);
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int t = 1; t <= S2; ++t) {
        const float4 q = *reinterpret_cast<const float4 *>(base + (int64_t)t * ldh);
        s.x += q.x;
        s.y += q.y;
        s.z += q.z;
        s.w += q.w;
    }
    const float inv = 1.0f / (float)S2;
    float *o = c2 + (int64_t)b * (2 * ldh);
    *reinterpret_cast<float4 *>(o + c) = self;
    *reinterpret_cast<float4 *>(o + ldh + c) = make_float4(s.x * inv, s.y * inv, s.z * inv, s.w * inv);
}

// dz1[m] = (instance 0: dc2[i][0 .. ldh); instance t > 0: dc2[i][ldh ..) / S2), switched off where h1[m] is zero
__global__ void k_sage_dz1(const float *__restrict__ dc2, const float *__restrict__ h1, int ldh, int B, int S2,
                           float *__restrict__ dz1) {
    const int quads = ldh / 4;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)B * (1 + S2) * quads) return;
    const int64_t m = i / quads;
    const int c = (int)(i % quads) * 4;
    const int b = (int)(m / (1 + S2)), t = (int)(m % (1 + S2));
    const float4 g = *reinterpret_cast<const float4 *>(dc2 + (int64_t)b * (2 * ldh) + (t == 0 ? 0 : ldh) + c);
    const float scale = t == 0 ? 1.0f : 1.0f / (float)S2;
    const float4 h = *reinterpret_cast<const float4 *>(h1 + m * ldh + c);
    float4 o;
    o.x = h.x > 0.0f ? g.x * scale : 0.0f;
    o.y = h.y > 0.0f ? g.y * scale : 0.0f;
    o.z = h.z > 0.0f ? g.z * scale : 0.0f;
    o.w = h.w > 0.0f ? g.w * scale : 0.0f;
    *reinterpret_cast<float4 *>(dz1 + m * ldh + c) = o;
}

__global__ void k_sage_ones(float *__restrict__ ones, uint8_t *__restrict__ mask, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        ones[i] = 1.0f;
        mask[i] = 1;
    }
}

// Copies the batch; an entry outside [0, n) becomes -1 (a vertex without features) and raises the sticky flag.
__global__ void k_sage_take_batch(const int32_t *__restrict__ batch, int B, int64_t n, int32_t *__restrict__ own,
                                  int32_t *flag) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B) return;
    int v = batch[i];
    if (v < 0 || v >= n) {
        v = -1;
        atomicOr(flag, 1);
    }
    own[i] = v;
}

bool aligned(const void *p) { return ((uintptr_t)p & 255u) == 0; }

}  // namespace

struct gcn_sage {
    const gcn_graph *g = nullptr;
    int f = 0, ldf = 0, hidden = 0, ldh = 0, classes = 0, ldc = 0, s1 = 0, s2 = 0, max_batch = 0;
    uint64_t seed = 0;
    int n_batch = 0;
    int64_t adam_steps = 0;
    bool have_forward = false, have_loss = false, have_backward = false;
    int32_t *batch = nullptr, *inner = nullptr, *nodes1 = nullptr, *outer = nullptr, *labels_b = nullptr, *flag = nullptr;
    float *c1 = nullptr, *h1 = nullptr, *c2 = nullptr, *logits = nullptr, *dz2 = nullptr, *dc2 = nullptr, *dz1 = nullptr;
    float *w1 = nullptr, *dw1 = nullptr, *m1 = nullptr, *v1 = nullptr, *w2 = nullptr, *dw2 = nullptr, *m2 = nullptr,
          *v2 = nullptr;
    float *ones = nullptr;
    uint8_t *mask = nullptr;
    float *partials = nullptr;
    size_t partial_floats = 0;
    double *loss_part = nullptr;
    long long *corr_part = nullptr;
    float *result = nullptr;
    long long *result_correct = nullptr;
};

namespace {

void carve_sage(Carver &c, gcn_sage &s) {
    const size_t B = (size_t)s.max_batch, n1 = B * (size_t)(1 + s.s2);
    s.batch = c.take<int32_t>(B);
    s.inner = c.take<int32_t>(B * s.s2);
    s.nodes1 = c.take<int32_t>(n1);
    s.outer = c.take<int32_t>(n1 * s.s1);
    s.labels_b = c.take<int32_t>(B);
    s.flag = c.take<int32_t>(16);
    s.c1 = c.take<float>(n1 * 2 * s.ldf);
    s.h1 = c.take<float>(n1 * s.ldh);
    s.c2 = c.take<float>(B * 2 * s.ldh);
    s.logits = c.take<float>(B * s.ldc);
    s.dz2 = c.take<float>(B * s.ldc);
    s.dc2 = c.take<float>(B * 2 * s.ldh);
    s.dz1 = c.take<float>(n1 * s.ldh);
    const size_t e1 = (size_t)2 * s.ldf * s.ldh, e2 = (size_t)2 * s.ldh * s.ldc;
    s.w1 = c.take<float>(e1);
    s.dw1 = c.take<float>(e1);
    s.m1 = c.take<float>(e1);
    s.v1 = c.take<float>(e1);
    s.w2 = c.take<float>(e2);
    s.dw2 = c.take<float>(e2);
    s.m2 = c.take<float>(e2);
    s.v2 = c.take<float>(e2);
    s.ones = c.take<float>(B);
    s.mask = c.take<uint8_t>(B);
    size_t pf = gemm_tn_partial_floats((int64_t)n1, 2 * s.ldf, s.ldh);
    const size_t pf2 = gemm_tn_partial_floats((int64_t)B, 2 * s.ldh, s.ldc);
    const size_t pf3 = gemm_nn_splitk_partial_floats((int64_t)n1, 2 * s.ldf, s.ldh);
    pf = pf > pf2 ? pf : pf2;
    s.partial_floats = pf > pf3 ? pf : pf3;
    s.partials = c.take<float>(s.partial_floats);
    s.loss_part = c.take<double>(kLossBlocks);
    s.corr_part = c.take<long long>(kLossBlocks);
    s.result = c.take<float>(4);
    s.result_correct = c.take<long long>(2);
}

int check_shape(const gcn_graph *g, int32_t hidden, int32_t s1, int32_t s2, int32_t max_batch) {
    if (!g || hidden < 1 || hidden > 256 || s1 < 1 || s1 > 1024 || s2 < 1 || s2 > 1024 || max_batch < 1 ||
        max_batch > 65536) {
        set_error("GraphSAGE: need a graph, 1 <= hidden <= 256, 1 <= S1, S2 <= 1024, 1 <= batch <= 65536");
        return GCN_EINVAL;
    }
    if (g->store_dtype != GCN_F32) {
        set_error("GraphSAGE: the graph must keep its features as float32");
        return GCN_EINVAL;
    }
    if (g->n_classes > 256) {
        set_error("GraphSAGE: at most 256 classes");
        return GCN_EINVAL;
    }
    return GCN_OK;
}

void fill_shape(gcn_sage &s, const gcn_graph *g, int32_t hidden, int32_t s1, int32_t s2, int32_t max_batch) {
    s.g = g;
    s.f = g->f;
    s.ldf = g->ldf;
    s.hidden = hidden;
    s.ldh = padded_width(hidden);
    s.classes = g->n_classes;
    s.ldc = padded_width(g->n_classes);
    s.s1 = s1;
    s.s2 = s2;
    s.max_batch = max_batch;
}

}  // namespace

extern "C" {

int gcn_sage_workspace_bytes(const gcn_graph *g, int32_t hidden, int32_t s1, int32_t s2, int32_t max_batch,
                             size_t *bytes) {
    int rc = check_shape(g, hidden, s1, s2, max_batch);
    if (rc) return rc;
    if (!bytes) {
        set_error("gcn_sage_workspace_bytes: null pointer");
        return GCN_EINVAL;
    }
    gcn_sage s;
    fill_shape(s, g, hidden, s1, s2, max_batch);
    Carver c(nullptr);
    carve_sage(c, s);
    *bytes = c.bytes();
    return GCN_OK;
}

int gcn_sage_create(gcn_sage **out, const gcn_graph *g, int32_t hidden, int32_t s1, int32_t s2, int32_t max_batch,
                    uint64_t seed, void *workspace, size_t workspace_bytes, void *stream) {
    if (out) *out = nullptr;
    if (!out) {
        set_error("gcn_sage_create: null pointer");
        return GCN_EINVAL;
    }
    size_t need = 0;
    int rc = gcn_sage_workspace_bytes(g, hidden, s1, s2, max_batch, &need);
    if (rc) return rc;
    if (!workspace || !aligned(workspace) || workspace_bytes < need) {
        set_error("gcn_sage_create: workspace missing, misaligned or smaller than %zu bytes", need);
        return GCN_EWORKSPACE;
    }
    gcn_sage *s = new (std::nothrow) gcn_sage;
    if (!s) {
        set_error("out of host memory");
        return GCN_EINVAL;
    }
    fill_shape(*s, g, hidden, s1, s2, max_batch);
    s->seed = seed;
    Carver c(workspace);
    carve_sage(c, *s);
    if (c.bytes() != need) {
        set_error("gcn_sage_create: internal layout mismatch");
        delete s;
        return GCN_EINVAL;
    }
    hipStream_t st = (hipStream_t)stream;
    rc = fill_zero(workspace, need, st);   // weights, moments, padding columns start at zero
    if (!rc) {
        k_sage_ones<<<dim3(blocks_for(max_batch, kThreads)), dim3(kThreads), 0, st>>>(s->ones, s->mask, max_batch);
        if (hipGetLastError() != hipSuccess) {
            set_error("gcn_sage_create: kernel launch failed");
            rc = GCN_EHIP;
        }
    }
    if (rc) {
        delete s;
        return rc;
    }
    *out = s;
    return GCN_OK;
}

int gcn_sage_destroy(gcn_sage *s) {
    delete s;
    return GCN_OK;
}

int gcn_sage_set_weights(gcn_sage *s, const float *w1, const float *w2, void *stream) {
    if (!s || !w1 || !w2) {
        set_error("gcn_sage_set_weights: null pointer");
        return GCN_EINVAL;
    }
    hipStream_t st = (hipStream_t)stream;
    // caller layout: w1 [2 f x hidden] (rows 0 .. f-1 act on the vertex's own features, rows f .. 2f-1 on the mean),
    // w2 [2 hidden x classes] likewise; library layout: the two halves start at rows 0 and ldf (ldh), zero padded
    int rc = fill_zero(s->w1, (size_t)2 * s->ldf * s->ldh * sizeof(float), st);
    if (!rc) rc = fill_zero(s->w2, (size_t)2 * s->ldh * s->ldc * sizeof(float), st);
    if (!rc) rc = pad_rows(w1, s->f, s->hidden, s->w1, GCN_F32, s->ldh, nullptr, st);
    if (!rc) rc = pad_rows(w1 + (size_t)s->f * s->hidden, s->f, s->hidden, s->w1 + (size_t)s->ldf * s->ldh, GCN_F32, s->ldh, nullptr, st);
    if (!rc) rc = pad_rows(w2, s->hidden, s->classes, s->w2, GCN_F32, s->ldc, nullptr, st);
    if (!rc) rc = pad_rows(w2 + (size_t)s->hidden * s->classes, s->hidden, s->classes, s->w2 + (size_t)s->ldh * s->ldc, GCN_F32, s->ldc, nullptr, st);
    if (!rc) rc = fill_zero(s->m1, (size_t)2 * s->ldf * s->ldh * sizeof(float), st);
    if (!rc) rc = fill_zero(s->v1, (size_t)2 * s->ldf * s->ldh * sizeof(float), st);
    if (!rc) rc = fill_zero(s->m2, (size_t)2 * s->ldh * s->ldc * sizeof(float), st);
    if (!rc) rc = fill_zero(s->v2, (size_t)2 * s->ldh * s->ldc * sizeof(float), st);
    s->adam_steps = 0;
    s->have_forward = s->have_loss = s->have_backward = false;
    return rc;
}

int gcn_sage_forward(gcn_sage *s, const int32_t *batch, int32_t n_batch, uint64_t step, void *stream) {
    if (!s || !batch || n_batch < 1 || n_batch > s->max_batch) {
        set_error("gcn_sage_forward: null pointer or batch size outside [1, %d]", s ? s->max_batch : 0);
        return GCN_EINVAL;
    }
    hipStream_t st = (hipStream_t)stream;
    const gcn_graph *g = s->g;
    const int B = n_batch, S1 = s->s1, S2 = s->s2;
    const int64_t n1 = (int64_t)B * (1 + S2);
    s->have_forward = s->have_loss = s->have_backward = false;
    // the batch is copied (later calls read it) and checked on the device; the flag is read by gcn_sage_loss_acc
    k_sage_take_batch<<<dim3(blocks_for(B, kThreads)), dim3(kThreads), 0, st>>>(batch, B, g->n, s->batch, s->flag);
    GCN_LAUNCH_CHECK();
    int rc = GCN_OK;
    k_sage_sample<<<dim3(blocks_for((int64_t)B * S2, kThreads)), dim3(kThreads), 0, st>>>(
        g->pb.rowptr, g->pb.col, s->batch, B, S2, level_key(s->seed, step, 2), s->inner);
    GCN_LAUNCH_CHECK();
    k_sage_nodes1<<<dim3(blocks_for(n1, kThreads)), dim3(kThreads), 0, st>>>(s->batch, s->inner, B, S2, g->labels,
                                                                               s->nodes1, s->labels_b);
    GCN_LAUNCH_CHECK();
    k_sage_sample<<<dim3(blocks_for(n1 * S1, kThreads)), dim3(kThreads), 0, st>>>(
        g->pb.rowptr, g->pb.col, s->nodes1, n1, S1, level_key(s->seed, step, 1), s->outer);
    GCN_LAUNCH_CHECK();
    const int t_gather = timing_open(kTimeSageGather, 0, st);
    k_sage_concat1<<<dim3(blocks_for(n1 * (s->ldf / 4), kThreads)), dim3(kThreads), 0, st>>>(
        static_cast<const float *>(g->x), s->ldf, s->nodes1, s->outer, S1, n1, s->c1);
    timing_close(t_gather, st);
    GCN_LAUNCH_CHECK();
    // a few thousand rows against 1216 of shared dimension: split that dimension so that the chip fills
    rc = gemm_nn_splitk(s->c1, 2 * s->ldf, s->w1, s->ldh, s->h1, s->ldh, n1, 2 * s->ldf, s->ldh, true, s->partials,
                        s->partial_floats, st);
    if (rc) return rc;
    k_sage_concat2<<<dim3(blocks_for((int64_t)B * (s->ldh / 4), kThreads)), dim3(kThreads), 0, st>>>(s->h1, s->ldh, B, S2,
                                                                                                     s->c2);
    GCN_LAUNCH_CHECK();
    rc = gemm_nn(s->c2, 2 * s->ldh, s->w2, s->ldc, s->logits, s->ldc, B, 2 * s->ldh, s->ldc, nullptr, nullptr, st);
    if (rc) return rc;
    s->n_batch = B;
    s->have_forward = true;
    return GCN_OK;
}

int gcn_sage_loss_acc(gcn_sage *s, float *loss, float *acc, int64_t *correct, void *stream) {
    if (!s || !s->have_forward) {
        set_error("gcn_sage_loss_acc: call gcn_sage_forward first");
        return GCN_EINVAL;
    }
    hipStream_t st = (hipStream_t)stream;
    int rc = loss_forward(s->n_batch, s->classes, s->logits, s->ldc, s->labels_b, s->mask, s->ones, s->n_batch, s->dz2,
                          GCN_F32, s->ldc, s->loss_part, s->corr_part, s->result, s->result_correct, st);
    if (rc) return rc;
    s->have_loss = true;
    if (loss || acc || correct) {
        float host[2];
        long long hc = 0;
        int32_t bad = 0;
        GCN_HIP(hipMemcpyAsync(host, s->result, sizeof(host), hipMemcpyDeviceToHost, st));
        GCN_HIP(hipMemcpyAsync(&hc, s->result_correct, sizeof(hc), hipMemcpyDeviceToHost, st));
        GCN_HIP(hipMemcpyAsync(&bad, s->flag, sizeof(bad), hipMemcpyDeviceToHost, st));
        GCN_HIP(hipStreamSynchronize(st));
        if (bad) {
            rc = fill_zero(s->flag, sizeof(int32_t), st);
            if (rc) return rc;
            set_error("gcn_sage_loss_acc: a batch entry since the last check was outside [0, %lld)", (long long)s->g->n);
            return GCN_EINVAL;
        }
        if (loss) *loss = host[0];
        if (acc) *acc = host[1];
        if (correct) *correct = (int64_t)hc;
    }
    return GCN_OK;
}

int gcn_sage_backward(gcn_sage *s, void *stream) {
    if (!s || !s->have_loss) {
        set_error("gcn_sage_backward: call gcn_sage_loss_acc first");
        return GCN_EINVAL;
    }
    hipStream_t st = (hipStream_t)stream;
    const int B = s->n_batch, S2 = s->s2;
    const int64_t n1 = (int64_t)B * (1 + S2);
    int rc = gemm_tn(s->c2, 2 * s->ldh, s->dz2, s->ldc, s->dw2, s->ldc, B, 2 * s->ldh, s->ldc, s->partials,
                     s->partial_floats, st);
    if (rc) return rc;
    rc = gemm_nt(s->dz2, s->ldc, s->w2, s->ldc, s->dc2, 2 * s->ldh, B, s->ldc, 2 * s->ldh, nullptr, nullptr, 0, 1.0f, st);
    if (rc) return rc;
    k_sage_dz1<<<dim3(blocks_for(n1 * (s->ldh / 4), kThreads)), dim3(kThreads), 0, st>>>(s->dc2, s->h1, s->ldh, B, S2,
                                                                                           s->dz1);
    GCN_LAUNCH_CHECK();
    rc = gemm_tn(s->c1, 2 * s->ldf, s->dz1, s->ldh, s->dw1, s->ldh, n1, 2 * s->ldf, s->ldh, s->partials, s->partial_floats,
                 st);
    if (rc) return rc;
    s->have_backward = true;
    return GCN_OK;
}

int gcn_sage_adam_step(gcn_sage *s, float lr, float beta1, float beta2, float eps, void *stream) {
    if (!s || !s->have_backward) {
        set_error("gcn_sage_adam_step: call gcn_sage_backward first");
        return GCN_EINVAL;
    }
    hipStream_t st = (hipStream_t)stream;
    int rc = adam_update(s->w1, s->dw1, s->m1, s->v1, (size_t)2 * s->ldf * s->ldh, lr, beta1, beta2, eps,
                         s->adam_steps + 1, st);
    if (!rc)
        rc = adam_update(s->w2, s->dw2, s->m2, s->v2, (size_t)2 * s->ldh * s->ldc, lr, beta1, beta2, eps,
                         s->adam_steps + 1, st);
    if (rc) return rc;
    s->adam_steps += 1;
    s->have_forward = s->have_loss = s->have_backward = false;
    return GCN_OK;
}

int gcn_sage_get_tensor(gcn_sage *s, int which, void *dst, size_t dst_elems, void *stream) {
    if (!s || !dst) {
        set_error("gcn_sage_get_tensor: null pointer");
        return GCN_EINVAL;
    }
    hipStream_t st = (hipStream_t)stream;
    const int B = s->n_batch;
    const int64_t n1 = (int64_t)B * (1 + s->s2);
    auto need = [&](size_t elems) {
        if (dst_elems >= elems) return true;
        set_error("gcn_sage_get_tensor: destination holds %zu elements, %zu needed", dst_elems, elems);
        return false;
    };
    auto halves = [&](const float *src, int rows, int ld_rows, int cols, int ld) -> int {   // [2 rows x cols] out of two padded halves
        int rc = unpad_rows(src, GCN_F32, ld, rows, cols, (float *)dst, nullptr, st);
        if (!rc) rc = unpad_rows(src + (size_t)ld_rows * ld, GCN_F32, ld, rows, cols, (float *)dst + (size_t)rows * cols, nullptr, st);
        return rc;
    };
    switch (which) {
        case GCN_SAGE_W1:
        case GCN_SAGE_DW1:
            if (which == GCN_SAGE_DW1 && !s->have_backward) break;
            if (!need((size_t)2 * s->f * s->hidden)) return GCN_EINVAL;
            return halves(which == GCN_SAGE_W1 ? s->w1 : s->dw1, s->f, s->ldf, s->hidden, s->ldh);
        case GCN_SAGE_W2:
        case GCN_SAGE_DW2:
            if (which == GCN_SAGE_DW2 && !s->have_backward) break;
            if (!need((size_t)2 * s->hidden * s->classes)) return GCN_EINVAL;
            return halves(which == GCN_SAGE_W2 ? s->w2 : s->dw2, s->hidden, s->ldh, s->classes, s->ldc);
        case GCN_SAGE_H1:
            if (!s->have_forward) break;
            if (!need((size_t)n1 * s->hidden)) return GCN_EINVAL;
            return unpad_rows(s->h1, GCN_F32, s->ldh, n1, s->hidden, (float *)dst, nullptr, st);
        case GCN_SAGE_LOGITS:
            if (!s->have_forward) break;
            if (!need((size_t)B * s->classes)) return GCN_EINVAL;
            return unpad_rows(s->logits, GCN_F32, s->ldc, B, s->classes, (float *)dst, nullptr, st);
        case GCN_SAGE_C1_MEAN:   // the aggregated half of layer 1's input: [n1 x f]
            if (!s->have_forward) break;
            if (!need((size_t)n1 * s->f)) return GCN_EINVAL;
            return unpad_rows(s->c1 + s->ldf, GCN_F32, 2 * s->ldf, n1, s->f, (float *)dst, nullptr, st);
        case GCN_SAGE_INNER:
            if (!s->have_forward) break;
            if (!need((size_t)B * s->s2)) return GCN_EINVAL;
            GCN_HIP(hipMemcpyAsync(dst, s->inner, (size_t)B * s->s2 * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
            return GCN_OK;
        case GCN_SAGE_OUTER:
            if (!s->have_forward) break;
            if (!need((size_t)n1 * s->s1)) return GCN_EINVAL;
            GCN_HIP(hipMemcpyAsync(dst, s->outer, (size_t)n1 * s->s1 * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
            return GCN_OK;
        default:
            set_error("gcn_sage_get_tensor: unknown tensor %d", which);
            return GCN_EINVAL;
    }
    set_error("gcn_sage_get_tensor: tensor %d is not available now", which);
    return GCN_EINVAL;
}

}  // extern "C"

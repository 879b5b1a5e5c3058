// Layout copies, the masked softmax cross-entropy with accuracy, and the SGD update.
//
// Task and metric: vertex classification scored by micro-F1, i.e. accuracy for one label per
// vertex (Section 2.2).  The paper does not print its loss; this is the softmax cross-entropy of
// the cited Kipf-Welling model, averaged over the train mask.  Update: plain SGD.
#include <cmath>

#include "common.hpp"
#include "dtypes.hpp"

namespace gcn {

namespace {

constexpr int kThreads = 256;

template <typename TDst>
__global__ void k_pad_rows(const float *__restrict__ src, int64_t rows, int width, TDst *__restrict__ dst, int ld,
                           const float *__restrict__ rowscale) {
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = rows * ld;
    if (t >= total) return;
    int64_t r = t / ld;
    int c = (int)(t - r * ld);
    float v = c < width ? src[r * width + c] : 0.0f;
    if (rowscale) v *= rowscale[r];
    dst[t] = narrow<TDst>(v);
}

template <typename TSrc>
__global__ void k_unpad_rows(const TSrc *__restrict__ src, int ld, int64_t rows, int width, float *__restrict__ dst,
                             const float *__restrict__ rowdiv) {
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = rows * width;
    if (t >= total) return;
    int64_t r = t / width;
    int c = (int)(t - r * width);
    float v = widen(src[r * ld + c]);
    if (rowdiv) v /= rowdiv[r];
    dst[t] = v;
}

template <typename T>
__global__ void k_scale_rows(const T *__restrict__ src, T *__restrict__ dst, int64_t rows, int ld,
                             const float *__restrict__ rowscale) {
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= rows * ld) return;
    dst[t] = narrow<T>(widen(src[t]) * rowscale[t / ld]);
}

__global__ void k_fill_zero(uint32_t *__restrict__ p, size_t words) {
    size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; t < words; t += stride) p[t] = 0u;
}

// One wave per vertex, waves stride over the vertices in a fixed pattern, so every partial sum
// is made of the same terms in the same order on every run.
template <typename TDz>
__global__ __launch_bounds__(kThreads) void k_loss(int64_t n, int classes, const float *__restrict__ logits, int ld,
                                                   const int32_t *__restrict__ labels,
                                                   const uint8_t *__restrict__ mask, const float *__restrict__ dinv,
                                                   float inv_ntrain, TDz *__restrict__ dzs, int ld_dz,
                                                   double *__restrict__ loss_part,
                                                   long long *__restrict__ corr_part) {
    __shared__ double s_loss[kThreads / 64];
    __shared__ long long s_corr[kThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t waves_total = (int64_t)gridDim.x * (kThreads / 64);
    double my_loss = 0.0;
    long long my_corr = 0;
    for (int64_t v = (int64_t)blockIdx.x * (kThreads / 64) + wave; v < n; v += waves_total) {
        const float *z = logits + v * ld;
        TDz *g = dzs + v * ld_dz;
        if (!mask[v]) {
            for (int c = lane; c < classes; c += 64) g[c] = narrow<TDz>(0.0f);
            continue;
        }
        // maximum and its lowest index
        float m = -INFINITY;
        int arg = 0x7fffffff;
        for (int c = lane; c < classes; c += 64) {
            float x = z[c];
            if (x > m) {
                m = x;
                arg = c;
            }
        }
#pragma unroll
        for (int d = 32; d > 0; d >>= 1) {
            float om = __shfl_xor(m, d, 64);
            int oa = __shfl_xor(arg, d, 64);
            if (om > m || (om == m && oa < arg)) {
                m = om;
                arg = oa;
            }
        }
        float s = 0.0f;
        for (int c = lane; c < classes; c += 64) s += expf(z[c] - m);
#pragma unroll
        for (int d = 32; d > 0; d >>= 1) s += __shfl_xor(s, d, 64);
        const float lse = m + logf(s);
        const int y = labels[v];
        const float scale = dinv[v] * inv_ntrain;
        for (int c = lane; c < classes; c += 64) {
            float p = expf(z[c] - lse);
            g[c] = narrow<TDz>((p - (c == y ? 1.0f : 0.0f)) * scale);
        }
        if (lane == 0) {
            my_loss += (double)(lse - z[y]);
            my_corr += (arg == y) ? 1 : 0;
        }
    }
    if (lane == 0) {
        s_loss[wave] = my_loss;
        s_corr[wave] = my_corr;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double a = 0.0;
        long long c = 0;
        for (int w = 0; w < kThreads / 64; ++w) {
            a += s_loss[w];
            c += s_corr[w];
        }
        loss_part[blockIdx.x] = a;
        corr_part[blockIdx.x] = c;
    }
}

// The same for at most 64 classes: a group of 16 lanes per vertex (four vertices per wave at a time), each lane
// holding up to four logits in registers, so a vertex costs one pass over its row and two 4-step reductions.
template <typename TDz>
__global__ __launch_bounds__(kThreads) void k_loss_small(int64_t n, int classes, const float *__restrict__ logits,
                                                         int ld, const int32_t *__restrict__ labels,
                                                         const uint8_t *__restrict__ mask,
                                                         const float *__restrict__ dinv, float inv_ntrain,
                                                         TDz *__restrict__ dzs, int ld_dz,
                                                         double *__restrict__ loss_part,
                                                         long long *__restrict__ corr_part, PlaneSink sink) {
    constexpr int kLanes = 16, kPerLane = 4;
    __shared__ double s_loss[kThreads / 64];
    __shared__ long long s_corr[kThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane % kLanes, grp = lane / kLanes;
    const int64_t groups_total = (int64_t)gridDim.x * (kThreads / kLanes);
    double my_loss = 0.0;
    long long my_corr = 0;
    // With a sink the gradient also goes out in the order the tile product of the backward aggregation reads it
    // (tiles.hip: rows 32 ct + 8 kg + 4 half + 0..3 of column c are the 16 bytes at units[((ct * 4 + kg) * 2 + half) *
    // ld + c]).  The four vertices of a wave are four consecutive rows (the group count is a multiple of four), so
    // lane (group, sub) writes element `group` of the unit of column sub + 16 i: a wave's store is 256 contiguous
    // bytes.  Rows from n up to the last whole block of 32 are written as zero.
    float *units = static_cast<float *>(sink.planes);
    const int64_t v_end = units ? (int64_t)sink.n_ct * 32 : n;
    auto to_units = [&](int64_t v, int c, float x) {
        if (units && c < sink.ld)
            units[((((v >> 5) * 4 + ((v >> 3) & 3)) * 2 + ((v >> 2) & 1)) * sink.ld + c) * 4 + (v & 3)] = x;
    };
    for (int64_t v = ((int64_t)blockIdx.x * (kThreads / 64) + wave) * (64 / kLanes) + grp; v < v_end; v += groups_total) {
        if (v >= n || !mask[v]) {
#pragma unroll
            for (int i = 0; i < kPerLane; ++i) {
                if (v < n && sub + kLanes * i < classes) dzs[v * ld_dz + sub + kLanes * i] = narrow<TDz>(0.0f);
                to_units(v, sub + kLanes * i, 0.0f);
            }
            continue;
        }
        const float *z = logits + v * ld;
        TDz *g = dzs + v * ld_dz;
        float x[kPerLane];
        float m = -INFINITY;
        int arg = 0x7fffffff;
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            const int c = sub + kLanes * i;
            x[i] = c < classes ? z[c] : -INFINITY;
            if (x[i] > m) {   // ascending c: the lowest index of the maximum
                m = x[i];
                arg = c;
            }
        }
#pragma unroll
        for (int d = kLanes / 2; d > 0; d >>= 1) {
            const float om = __shfl_xor(m, d, 64);
            const int oa = __shfl_xor(arg, d, 64);
            if (om > m || (om == m && oa < arg)) {
                m = om;
                arg = oa;
            }
        }
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < kPerLane; ++i)
            if (sub + kLanes * i < classes) s += expf(x[i] - m);
#pragma unroll
        for (int d = kLanes / 2; d > 0; d >>= 1) s += __shfl_xor(s, d, 64);
        const float lse = m + logf(s);
        const int y = labels[v];
        const float scale = dinv[v] * inv_ntrain;
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            const int c = sub + kLanes * i;
            float gv = 0.0f;
            if (c < classes) {
                const TDz stored = narrow<TDz>((expf(x[i] - lse) - (c == y ? 1.0f : 0.0f)) * scale);
                g[c] = stored;
                gv = widen(stored);
            }
            to_units(v, c, gv);
        }
        if (sub == 0) {
            my_loss += (double)(lse - z[y]);
            my_corr += (arg == y) ? 1 : 0;
        }
    }
    // the four group leaders of the wave, in a fixed order
#pragma unroll
    for (int d = kLanes; d < 64; d <<= 1) {
        my_loss += __shfl_xor(my_loss, d, 64);
        my_corr += __shfl_xor(my_corr, d, 64);
    }
    if (lane == 0) {
        s_loss[wave] = my_loss;
        s_corr[wave] = my_corr;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double a = 0.0;
        long long c = 0;
        for (int w = 0; w < kThreads / 64; ++w) {
            a += s_loss[w];
            c += s_corr[w];
        }
        loss_part[blockIdx.x] = a;
        corr_part[blockIdx.x] = c;
    }
}

__global__ __launch_bounds__(kThreads) void k_loss_final(int parts, const double *__restrict__ loss_part,
                                                         const long long *__restrict__ corr_part, double inv_ntrain,
                                                         float *__restrict__ result,
                                                         long long *__restrict__ result_correct) {
    __shared__ double s_loss[kThreads];
    __shared__ long long s_corr[kThreads];
    double a = 0.0;
    long long c = 0;
    for (int p = threadIdx.x; p < parts; p += kThreads) {
        a += loss_part[p];
        c += corr_part[p];
    }
    s_loss[threadIdx.x] = a;
    s_corr[threadIdx.x] = c;
    __syncthreads();
    for (int d = kThreads / 2; d > 0; d >>= 1) {
        if (threadIdx.x < d) {
            s_loss[threadIdx.x] += s_loss[threadIdx.x + d];
            s_corr[threadIdx.x] += s_corr[threadIdx.x + d];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        result[0] = (float)(s_loss[0] * inv_ntrain);
        result[1] = (float)((double)s_corr[0] * inv_ntrain);
        *result_correct = s_corr[0];
    }
}

// Which XCD each workgroup of a launch runs on: the XCC_ID hardware register (low 4 bits), read with s_getreg.
__global__ void k_xcc_ids(int32_t *__restrict__ out) {
    if (threadIdx.x == 0) out[blockIdx.x] = (int32_t)(__builtin_amdgcn_s_getreg((3 << 11) | 20) & 0xf);
}

// Plain streaming copy of 16-byte words: the known-size kernel hardware byte counters are scaled by.
__global__ void k_calibration_copy(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t words) {
    size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < words) dst[t] = src[t];
}

// All layers in one launch: element t of the concatenation belongs to the first layer whose end is beyond it.
__global__ void k_sgd(SgdLayers ls, float lr) {
    const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t first = 0;
    for (int l = 0; l < ls.n; ++l) {
        if (t < ls.end[l]) {
            ls.w[l][t - first] = ls.w[l][t - first] - lr * ls.dw[l][t - first];
            return;
        }
        first = ls.end[l];
    }
}

// Adam (Kingma & Ba): c1 = 1 - beta1^t, c2 = 1 - beta2^t are formed on the host in double precision.
__global__ void k_adam(float *__restrict__ w, const float *__restrict__ dw, float *__restrict__ m,
                       float *__restrict__ v, size_t count, float lr, float beta1, float beta2, float eps,
                       float inv_c1, float inv_c2) {
    size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= count) return;
    const float g = dw[t];
    const float mt = beta1 * m[t] + (1.0f - beta1) * g;
    const float vt = beta2 * v[t] + (1.0f - beta2) * g * g;
    m[t] = mt;
    v[t] = vt;
    w[t] = w[t] - lr * (mt * inv_c1) / (sqrtf(vt * inv_c2) + eps);
}

// dst[t] = (1 / count) * sum over the models, in list order, of srcs[i][t]; then every model gets dst.
struct AverageList {
    float *w[64];
    int count;
};
__global__ void k_average(AverageList list, size_t elems) {
    size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= elems) return;
    float s = 0.0f;
    for (int i = 0; i < list.count; ++i) s += list.w[i][t];
    s *= 1.0f / (float)list.count;
    for (int i = 0; i < list.count; ++i) list.w[i][t] = s;
}

// bfloat16 copies of a weight matrix w [rows x ld]: wb in the same layout, wbt transposed [ld x ld_t]
__global__ void k_weight_copies(const float *__restrict__ w, int rows, int ld, bf16_t *__restrict__ wb,
                                bf16_t *__restrict__ wbt, int ld_t) {
    size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (size_t)rows * ld) return;
    const int r = (int)(t / ld), c = (int)(t % ld);
    const bf16_t v = (bf16_t)w[t];
    wb[t] = v;
    wbt[(size_t)c * ld_t + r] = v;
}

inline unsigned blocks_for(int64_t items, int per_block) { return (unsigned)((items + per_block - 1) / per_block); }

}  // namespace

int pad_rows(const float *src, int64_t rows, int width, void *dst, int dst_dtype, int ld, const float *rowscale,
             hipStream_t st) {
    if (rows <= 0) return GCN_OK;
    const dim3 grid(blocks_for(rows * ld, kThreads));
    if (dst_dtype == GCN_BF16)
        k_pad_rows<bf16_t><<<grid, dim3(kThreads), 0, st>>>(src, rows, width, (bf16_t *)dst, ld, rowscale);
    else
        k_pad_rows<float><<<grid, dim3(kThreads), 0, st>>>(src, rows, width, (float *)dst, ld, rowscale);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int unpad_rows(const void *src, int src_dtype, int ld, int64_t rows, int width, float *dst, const float *rowdiv,
               hipStream_t st) {
    if (rows <= 0) return GCN_OK;
    const dim3 grid(blocks_for(rows * width, kThreads));
    if (src_dtype == GCN_BF16)
        k_unpad_rows<bf16_t><<<grid, dim3(kThreads), 0, st>>>((const bf16_t *)src, ld, rows, width, dst, rowdiv);
    else
        k_unpad_rows<float><<<grid, dim3(kThreads), 0, st>>>((const float *)src, ld, rows, width, dst, rowdiv);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int scale_rows(const void *src, void *dst, int dtype, int64_t rows, int ld, const float *rowscale, hipStream_t st) {
    if (rows <= 0) return GCN_OK;
    const dim3 grid(blocks_for(rows * ld, kThreads));
    if (dtype == GCN_BF16)
        k_scale_rows<bf16_t><<<grid, dim3(kThreads), 0, st>>>((const bf16_t *)src, (bf16_t *)dst, rows, ld, rowscale);
    else
        k_scale_rows<float><<<grid, dim3(kThreads), 0, st>>>((const float *)src, (float *)dst, rows, ld, rowscale);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int weight_copies(const float *w, int rows, int ld, void *wb, void *wbt, int ld_t, hipStream_t st) {
    k_weight_copies<<<dim3(blocks_for((int64_t)rows * ld, kThreads)), dim3(kThreads), 0, st>>>(
        w, rows, ld, (bf16_t *)wb, (bf16_t *)wbt, ld_t);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int fill_zero(void *p, size_t bytes, hipStream_t st) {
    if (bytes == 0) return GCN_OK;
    if (bytes % 4 != 0) {
        set_error("fill_zero: size not a multiple of 4");
        return GCN_EINVAL;
    }
    size_t words = bytes / 4;
    unsigned blocks = (unsigned)((words + kThreads - 1) / kThreads);
    if (blocks > 65536u) blocks = 65536u;
    k_fill_zero<<<dim3(blocks), dim3(kThreads), 0, st>>>((uint32_t *)p, words);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

bool loss_can_sink(int classes, int dz_dtype) { return classes <= 64 && dz_dtype == GCN_F32; }

int loss_forward(int64_t n, int classes, const float *logits, int ld, const int32_t *labels, const uint8_t *mask,
                 const float *dinv, int64_t n_train, void *dzs, int dz_dtype, int ld_dz, double *loss_part,
                 long long *corr_part, float *result, long long *result_correct, hipStream_t st,
                 const PlaneSink *sink) {
    const PlaneSink none{nullptr, 0, 0};
    const bool sinks = sink && sink->planes && loss_can_sink(classes, dz_dtype);
    int blocks = (int)(classes <= 64 ? (n + 15) / 16 + 2 : (n + 3) / 4);   // (+ 2: the rows up to a whole block of 32)
    if (blocks > kLossBlocks) blocks = kLossBlocks;
    if (blocks < 1) blocks = 1;
    const float inv = (float)(1.0 / (double)n_train);
    if (classes <= 64 && dz_dtype == GCN_BF16)
        k_loss_small<bf16_t><<<dim3(blocks), dim3(kThreads), 0, st>>>(n, classes, logits, ld, labels, mask, dinv, inv,
                                                                      (bf16_t *)dzs, ld_dz, loss_part, corr_part, none);
    else if (classes <= 64)
        k_loss_small<float><<<dim3(blocks), dim3(kThreads), 0, st>>>(n, classes, logits, ld, labels, mask, dinv, inv,
                                                                     (float *)dzs, ld_dz, loss_part, corr_part,
                                                                     sinks ? *sink : none);
    else if (dz_dtype == GCN_BF16)
        k_loss<bf16_t><<<dim3(blocks), dim3(kThreads), 0, st>>>(n, classes, logits, ld, labels, mask, dinv, inv,
                                                                (bf16_t *)dzs, ld_dz, loss_part, corr_part);
    else
        k_loss<float><<<dim3(blocks), dim3(kThreads), 0, st>>>(n, classes, logits, ld, labels, mask, dinv, inv,
                                                               (float *)dzs, ld_dz, loss_part, corr_part);
    GCN_LAUNCH_CHECK();
    k_loss_final<<<dim3(1), dim3(kThreads), 0, st>>>(blocks, loss_part, corr_part, 1.0 / (double)n_train, result,
                                                     result_correct);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int adam_update(float *w, const float *dw, float *m, float *v, size_t count, float lr, float beta1, float beta2,
                float eps, int64_t step, hipStream_t st) {
    if (count == 0) return GCN_OK;
    if (step < 1 || !(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f) || !(eps > 0.0f)) {
        set_error("adam: step must be >= 1, betas in [0, 1), eps > 0");
        return GCN_EINVAL;
    }
    const double c1 = 1.0 - std::pow((double)beta1, (double)step), c2 = 1.0 - std::pow((double)beta2, (double)step);
    k_adam<<<dim3(blocks_for((int64_t)count, kThreads)), dim3(kThreads), 0, st>>>(
        w, dw, m, v, count, lr, beta1, beta2, eps, (float)(1.0 / c1), (float)(1.0 / c2));
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int average_in_place(float *const *weights, int count, size_t elems, hipStream_t st) {
    if (count < 1 || count > 64) {
        set_error("parameter averaging: between 1 and 64 models");
        return GCN_EINVAL;
    }
    if (elems == 0) return GCN_OK;
    AverageList list;
    list.count = count;
    for (int i = 0; i < count; ++i) list.w[i] = weights[i];
    k_average<<<dim3(blocks_for((int64_t)elems, kThreads)), dim3(kThreads), 0, st>>>(list, elems);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int xcc_ids(int32_t *out, int n_blocks, hipStream_t st) {
    if (n_blocks <= 0) return GCN_OK;
    k_xcc_ids<<<dim3(n_blocks), dim3(kThreads), 0, st>>>(out);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int calibration_copy(const void *src, void *dst, size_t bytes, hipStream_t st) {
    if (bytes % 16 != 0 || bytes == 0 || bytes / 16 > 0x7fffffffull * 256ull) {
        set_error("calibration copy: size must be a positive multiple of 16 bytes");
        return GCN_EINVAL;
    }
    const size_t words = bytes / 16;
    k_calibration_copy<<<dim3((unsigned)((words + kThreads - 1) / kThreads)), dim3(kThreads), 0, st>>>(
        (const uint4 *)src, (uint4 *)dst, words);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int sgd_update(const SgdLayers &ls, float lr, hipStream_t st) {
    if (ls.n < 1 || ls.n > kMaxLayers) {
        set_error("sgd_update: %d layers", ls.n);
        return GCN_EINVAL;
    }
    const size_t total = ls.end[ls.n - 1];
    if (total == 0) return GCN_OK;
    k_sgd<<<dim3(blocks_for((int64_t)total, kThreads)), dim3(kThreads), 0, st>>>(ls, lr);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

}  // namespace gcn

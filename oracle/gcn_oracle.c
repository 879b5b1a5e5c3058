/*
 * CPU oracle for the full-batch Kipf-Welling GCN training step on one partition.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * GPU library must compute; it is called by the tests, by the smoke check and by the
 * benchmark's CPU-baseline leg, and by nothing else.  It shares no code, header,
 * table or helper with the GPU path.  All floating point is fp64.
 *
 * What it follows:
 *   - layer rule H^L = sigma(A_hat H^{L-1} W^L), H^0 = X          (Section 4.1)
 *   - inputs: feature matrix X with one row per vertex, adjacency A  (Section 2.1)
 *   - A_hat is the "normalized adjacency matrix" of the footnote to Section 4.1,
 *     taken in the form of the cited Kipf-Welling model:
 *     A_hat = D^-1/2 (A + I) D^-1/2 with D the row sums of A + I, A binary
 *   - task: vertex classification scored by micro-F1, which for one label per
 *     vertex is plain accuracy                                      (Section 2.2)
 *   - cost model O(L nnz(A) F + L N F^2): one sparse product and one dense product
 *     per layer                                                     (Section 5.4)
 * Readings where the paper is silent (sigma = ReLU on hidden layers, linear last
 * layer, softmax cross-entropy averaged over the train mask, no bias, plain SGD,
 * lowest index wins argmax ties) are listed in the design notes of the repository.
 *
 * Loops are the definitions written out.  OpenMP, where used, gives each output row
 * to exactly one thread, so results do not depend on the thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_EINVAL (-1)
#define ORC_EGRAPH (-2)
#define ORC_ELABEL (-3)

static int cmp_i32(const void *a, const void *b) {
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* ---------------------------------------------------------------- step 1: canonical A + I
 * Row i of the canonical pattern is the ascending list of distinct j with A_ij != 0,
 * j != i, together with i itself: exactly one self-loop of weight one, whether or not
 * the raw input already had one, and repeated entries count once.
 * Phase "count": deg[i] = length of canonical row i  (the diagonal of D).
 * Phase "fill" : writes the columns at out_rowptr[i].
 */
static int64_t canonical_row(int64_t i, const int64_t *rowptr, const int32_t *col, int32_t *tmp) {
    int64_t b = rowptr[i], e = rowptr[i + 1], m = 0;
    for (int64_t p = b; p < e; ++p)
        if (col[p] != (int32_t)i) tmp[m++] = col[p];
    tmp[m++] = (int32_t)i;
    qsort(tmp, (size_t)m, sizeof(int32_t), cmp_i32);
    int64_t k = 0;
    for (int64_t p = 0; p < m; ++p)
        if (p == 0 || tmp[p] != tmp[p - 1]) tmp[k++] = tmp[p];
    return k;
}

int orc_validate_csr(int64_t n, int64_t nnz, const int64_t *rowptr, const int32_t *col) {
    if (n <= 0 || rowptr[0] != 0 || rowptr[n] != nnz) return ORC_EGRAPH;
    for (int64_t i = 0; i < n; ++i)
        if (rowptr[i + 1] < rowptr[i]) return ORC_EGRAPH;
    for (int64_t p = 0; p < nnz; ++p)
        if (col[p] < 0 || col[p] >= n) return ORC_EGRAPH;
    return ORC_OK;
}

int orc_canonical_degrees(int64_t n, const int64_t *rowptr, const int32_t *col, int32_t *deg) {
    int64_t maxlen = 0;
    for (int64_t i = 0; i < n; ++i)
        if (rowptr[i + 1] - rowptr[i] > maxlen) maxlen = rowptr[i + 1] - rowptr[i];
    int bad = 0;
#pragma omp parallel
    {
        int32_t *tmp = (int32_t *)malloc((size_t)(maxlen + 1) * sizeof(int32_t));
        if (!tmp) {
#pragma omp atomic write
            bad = 1;
        } else {
#pragma omp for schedule(static)
            for (int64_t i = 0; i < n; ++i) deg[i] = (int32_t)canonical_row(i, rowptr, col, tmp);
            free(tmp);
        }
    }
    return bad ? ORC_EINVAL : ORC_OK;
}

int orc_canonical_fill(int64_t n, const int64_t *rowptr, const int32_t *col, const int64_t *out_rowptr,
                       int32_t *out_col) {
    int64_t maxlen = 0;
    for (int64_t i = 0; i < n; ++i)
        if (rowptr[i + 1] - rowptr[i] > maxlen) maxlen = rowptr[i + 1] - rowptr[i];
    int bad = 0;
#pragma omp parallel
    {
        int32_t *tmp = (int32_t *)malloc((size_t)(maxlen + 1) * sizeof(int32_t));
        if (!tmp) {
#pragma omp atomic write
            bad = 1;
        } else {
#pragma omp for schedule(static)
            for (int64_t i = 0; i < n; ++i) {
                int64_t k = canonical_row(i, rowptr, col, tmp);
                if (k != out_rowptr[i + 1] - out_rowptr[i]) {
#pragma omp atomic write
                    bad = 1;
                } else {
                    memcpy(out_col + out_rowptr[i], tmp, (size_t)k * sizeof(int32_t));
                }
            }
            free(tmp);
        }
    }
    return bad ? ORC_EINVAL : ORC_OK;
}

/* 1 if the canonical pattern is symmetric (j in row i  <=>  i in row j), else 0. */
int orc_is_symmetric(int64_t n, const int64_t *rowptr, const int32_t *col) {
    int ok = 1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            int32_t j = col[p], key = (int32_t)i;
            const int32_t *hit = (const int32_t *)bsearch(&key, col + rowptr[j], (size_t)(rowptr[j + 1] - rowptr[j]),
                                                          sizeof(int32_t), cmp_i32);
            if (!hit) {
#pragma omp atomic write
                ok = 0;
            }
        }
    }
    return ok;
}

/* ---------------------------------------------------------------- step 2: D^-1/2 */
void orc_dinv(int64_t n, const int64_t *rowptr, double *dinv) {
    for (int64_t i = 0; i < n; ++i) dinv[i] = 1.0 / sqrt((double)(rowptr[i + 1] - rowptr[i]));
}

/* ---------------------------------------------------------------- aggregation  Z = A_hat T
 * Z[i,:] = sum over j in canonical row i of  dinv_i * dinv_j * T[j,:],  in row order. */
void orc_aggregate(int64_t n, const int64_t *rowptr, const int32_t *col, const double *dinv, int64_t w,
                   const double *T, double *Z) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double *z = Z + i * w;
        for (int64_t c = 0; c < w; ++c) z[c] = 0.0;
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            int64_t j = col[p];
            double a = dinv[i] * dinv[j];
            const double *t = T + j * w;
            for (int64_t c = 0; c < w; ++c) z[c] += a * t[c];
        }
    }
}

/* ---------------------------------------------------------------- dense products, triple loops
 * nn: C[m x n] = A[m x k] B[k x n];  tn: C[m x n] = A[k x m]^T B[k x n];  nt: C[m x n] = A[m x k] B[n x k]^T.
 * For every C[i,j] the sum runs over the shared index in ascending order. */
void orc_matmul_nn(int64_t m, int64_t k, int64_t n, const double *A, const double *B, double *C) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        double *c = C + i * n;
        for (int64_t j = 0; j < n; ++j) c[j] = 0.0;
        for (int64_t p = 0; p < k; ++p) {
            double a = A[i * k + p];
            const double *b = B + p * n;
            for (int64_t j = 0; j < n; ++j) c[j] += a * b[j];
        }
    }
}

void orc_matmul_tn(int64_t m, int64_t k, int64_t n, const double *A, const double *B, double *C) {
#pragma omp parallel
    {
#pragma omp for schedule(static)
        for (int64_t i = 0; i < m; ++i)
            for (int64_t j = 0; j < n; ++j) C[i * n + j] = 0.0;
        /* each thread owns a fixed block of output rows i and walks p upward */
#pragma omp for schedule(static)
        for (int64_t ib = 0; ib < (m + 7) / 8; ++ib) {
            int64_t i0 = ib * 8, i1 = i0 + 8 < m ? i0 + 8 : m;
            for (int64_t p = 0; p < k; ++p) {
                const double *b = B + p * n;
                for (int64_t i = i0; i < i1; ++i) {
                    double a = A[p * m + i];
                    double *c = C + i * n;
                    for (int64_t j = 0; j < n; ++j) c[j] += a * b[j];
                }
            }
        }
    }
}

void orc_matmul_nt(int64_t m, int64_t k, int64_t n, const double *A, const double *B, double *C) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < n; ++j) {
            double s = 0.0;
            for (int64_t p = 0; p < k; ++p) s += A[i * k + p] * B[j * k + p];
            C[i * n + j] = s;
        }
}

/* ---------------------------------------------------------------- dropout mask (optional, p = 0 in all benchmarks)
 * keep(element) = [ top 32 bits of mix(seed, epoch, layer, element) >= floor(p * 2^32) ], a pure integer
 * function, so any implementation of the same mixer gives the same mask bit for bit.
 * mix = SplitMix64 finaliser applied to a key folded from the four integers. */
static uint64_t sm64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

void orc_dropout_keep(uint64_t seed, uint64_t epoch, uint64_t layer, int64_t rows, int64_t width, double p,
                      uint8_t *keep) {
    uint64_t thr = (uint64_t)floor(p * 4294967296.0);
    uint64_t key = sm64(sm64(seed) ^ (epoch * 0xD1B54A32D192ED03ULL) ^ (layer * 0x8CB92BA72F3D8DD7ULL));
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < width; ++c) {
            uint64_t e = (uint64_t)r * (uint64_t)width + (uint64_t)c;
            uint64_t h = sm64(key + e * 0x9E3779B97F4A7C15ULL);
            keep[r * width + c] = (uint8_t)((h >> 32) >= thr);
        }
}

/* ---------------------------------------------------------------- activation (hidden layers)
 * H = max(Z, 0), then, if keep != NULL, H *= keep / (1 - p). */
void orc_relu_dropout(int64_t count, const double *Z, const uint8_t *keep, double p, double *H) {
    double s = keep ? 1.0 / (1.0 - p) : 1.0;
    for (int64_t t = 0; t < count; ++t) {
        double h = Z[t] > 0.0 ? Z[t] : 0.0;
        H[t] = keep ? (keep[t] ? h * s : 0.0) : h;
    }
}

/* dZ = dH * [Z > 0] * keep / (1 - p) */
void orc_relu_dropout_backward(int64_t count, const double *Z, const uint8_t *keep, double p, const double *dH,
                               double *dZ) {
    double s = keep ? 1.0 / (1.0 - p) : 1.0;
    for (int64_t t = 0; t < count; ++t) {
        double g = Z[t] > 0.0 ? dH[t] : 0.0;
        dZ[t] = keep ? (keep[t] ? g * s : 0.0) : g;
    }
}

/* ---------------------------------------------------------------- loss, accuracy, dLoss/dlogits
 * Over masked vertices v: lse_v = m + log sum_c exp(z_vc - m), m = max_c z_vc;
 * loss = mean_v (lse_v - z_{v,y_v});  prediction = smallest c reaching the maximum;
 * dZ[v,c] = mask_v (exp(z_vc - lse_v) - [c == y_v]) / n_train.   dZ may be NULL. */
int orc_loss_acc(int64_t n, int64_t classes, const double *logits, const int32_t *labels, const uint8_t *mask,
                 double *loss, int64_t *correct, int64_t *n_train, double *dZ) {
    int64_t nt = 0, ok = 0;
    for (int64_t v = 0; v < n; ++v) {
        if (labels[v] < 0 || labels[v] >= classes) return ORC_ELABEL;
        if (mask[v]) ++nt;
    }
    *n_train = nt;
    if (nt == 0) return ORC_EINVAL;
    double total = 0.0;
    for (int64_t v = 0; v < n; ++v) {
        const double *z = logits + v * classes;
        if (!mask[v]) {
            if (dZ)
                for (int64_t c = 0; c < classes; ++c) dZ[v * classes + c] = 0.0;
            continue;
        }
        double m = z[0];
        int64_t arg = 0;
        for (int64_t c = 1; c < classes; ++c)
            if (z[c] > m) {
                m = z[c];
                arg = c;
            }
        double s = 0.0;
        for (int64_t c = 0; c < classes; ++c) s += exp(z[c] - m);
        double lse = m + log(s);
        total += lse - z[labels[v]];
        if (arg == labels[v]) ++ok;
        if (dZ)
            for (int64_t c = 0; c < classes; ++c)
                dZ[v * classes + c] = (exp(z[c] - lse) - (c == labels[v] ? 1.0 : 0.0)) / (double)nt;
    }
    *loss = total / (double)nt;
    *correct = ok;
    return ORC_OK;
}

/* ---------------------------------------------------------------- update  W <- W - lr dW */
void orc_sgd(int64_t count, double lr, const double *dW, double *W) {
    for (int64_t t = 0; t < count; ++t) W[t] -= lr * dW[t];
}

/* ---------------------------------------------------------------- Adam, the optimiser the paper trains KW-GCN with
 * (Section 4.1: Adam, learning rate 0.02; the other constants are not printed, the defaults of the Adam
 * paper are beta1 = 0.9, beta2 = 0.999, eps = 1e-8).  step counts from 1.
 *   m <- b1 m + (1 - b1) g ;  v <- b2 v + (1 - b2) g^2 ;  W <- W - lr (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps) */
void orc_adam(int64_t count, double lr, double beta1, double beta2, double eps, int64_t step, const double *dW,
              double *m, double *v, double *W) {
    double c1 = 1.0 - pow(beta1, (double)step), c2 = 1.0 - pow(beta2, (double)step);
    for (int64_t t = 0; t < count; ++t) {
        double g = dW[t];
        m[t] = beta1 * m[t] + (1.0 - beta1) * g;
        v[t] = beta2 * v[t] + (1.0 - beta2) * g * g;
        W[t] -= lr * (m[t] / c1) / (sqrt(v[t] / c2) + eps);
    }
}

/*
 * CPU oracle for the convolution-layer operators of the bi-graph (paper section 2, Figure 1(b):
 * operators are functions of their incoming tensors whose results go to the outgoing tensors).
 *
 * TEST INFRASTRUCTURE ONLY. Nothing in the product path may link or call this file; it shares no
 * code, header, table or helper with the HIP library.
 *
 * The paper defines the layer only by reference ("the convolution layer defined in Caffe"), so
 * each function below is the plain textbook definition written out as nested loops, with an fp64
 * accumulator per output element and inputs widened exactly to fp64:
 *   - cross-correlation (no kernel flip), dense NCHW / KCRS, zero padding, no dilation, one group;
 *   - output extent floor((in + 2*pad - k)/stride) + 1;
 *   - gradients are plain sums over the batch (no 1/N), which is what makes data-parallel shards
 *     additive (paper section 3.4).
 * Parallelism is OpenMP over independent outputs only, so no result depends on the thread count.
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int64_t N, C, H, W;   /* input  x[N][C][H][W]            */
    int64_t K, R, S;      /* filter w[K][C][R][S]            */
    int64_t sh, sw;       /* stride                          */
    int64_t ph, pw;       /* symmetric zero padding          */
} oracle_conv_shape;

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Output extent along one axis; -1 when the padded input is smaller than the kernel or the
 * arguments are not a legal convolution. */
int64_t oracle_out_extent(int64_t in, int64_t k, int64_t stride, int64_t pad) {
    if (in <= 0 || k <= 0 || stride <= 0 || pad < 0) return -1;
    if (in + 2 * pad < k) return -1;
    return (in + 2 * pad - k) / stride + 1;
}

#define XI(n, c, h, w_) ((((n) * g->C + (c)) * g->H + (h)) * g->W + (w_))
#define WI(k, c, r, s) ((((k) * g->C + (c)) * g->R + (r)) * g->S + (s))
#define YI(n, k, p, q) ((((n) * g->K + (k)) * P + (p)) * Q + (q))

/* y[n,k,p,q] = sum_{c,r,s} x[n,c,p*sh-ph+r,q*sw-pw+s] * w[k,c,r,s]; taps outside x are zero. */
void oracle_conv_fwd(const oracle_conv_shape* g, const float* x, const float* w, double* y) {
    const int64_t P = oracle_out_extent(g->H, g->R, g->sh, g->ph);
    const int64_t Q = oracle_out_extent(g->W, g->S, g->sw, g->pw);
    if (P <= 0 || Q <= 0) return;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < g->N; ++n)
        for (int64_t k = 0; k < g->K; ++k)
            for (int64_t p = 0; p < P; ++p)
                for (int64_t q = 0; q < Q; ++q) {
                    double acc = 0.0;
                    for (int64_t c = 0; c < g->C; ++c)
                        for (int64_t r = 0; r < g->R; ++r) {
                            const int64_t h = p * g->sh - g->ph + r;
                            if (h < 0 || h >= g->H) continue;
                            for (int64_t s = 0; s < g->S; ++s) {
                                const int64_t w_ = q * g->sw - g->pw + s;
                                if (w_ < 0 || w_ >= g->W) continue;
                                acc += (double)x[XI(n, c, h, w_)] * (double)w[WI(k, c, r, s)];
                            }
                        }
                    y[YI(n, k, p, q)] = acc;
                }
}

/* Bias operator: y[n,k,:,:] += b[k], in place on the fp64 tensor. */
void oracle_bias_fwd(double* y, const float* b, int64_t N, int64_t K, int64_t PQ) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            double* row = y + (n * K + k) * PQ;
            for (int64_t i = 0; i < PQ; ++i) row[i] += (double)b[k];
        }
}

/* Backward-data in SCATTER form: every (n,k,p,q,c,r,s) product that the forward pass formed is
 * pushed back onto the input position it read. dx must hold N*C*H*W doubles; it is overwritten. */
void oracle_conv_bwd_data(const oracle_conv_shape* g, const float* dy, const float* w, double* dx) {
    const int64_t P = oracle_out_extent(g->H, g->R, g->sh, g->ph);
    const int64_t Q = oracle_out_extent(g->W, g->S, g->sw, g->pw);
    memset(dx, 0, sizeof(double) * (size_t)(g->N * g->C * g->H * g->W));
    if (P <= 0 || Q <= 0) return;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < g->N; ++n) /* images are independent: no two threads share a dx row */
        for (int64_t k = 0; k < g->K; ++k)
            for (int64_t p = 0; p < P; ++p)
                for (int64_t q = 0; q < Q; ++q) {
                    const double gy = (double)dy[YI(n, k, p, q)];
                    for (int64_t c = 0; c < g->C; ++c)
                        for (int64_t r = 0; r < g->R; ++r) {
                            const int64_t h = p * g->sh - g->ph + r;
                            if (h < 0 || h >= g->H) continue;
                            for (int64_t s = 0; s < g->S; ++s) {
                                const int64_t w_ = q * g->sw - g->pw + s;
                                if (w_ < 0 || w_ >= g->W) continue;
                                dx[XI(n, c, h, w_)] += gy * (double)w[WI(k, c, r, s)];
                            }
                        }
                }
}

static double dw_element(const oracle_conv_shape* g, const float* x, const float* dy,
                         int64_t P, int64_t Q, int64_t k, int64_t c, int64_t r, int64_t s) {
    double acc = 0.0;
    for (int64_t n = 0; n < g->N; ++n)
        for (int64_t p = 0; p < P; ++p) {
            const int64_t h = p * g->sh - g->ph + r;
            if (h < 0 || h >= g->H) continue;
            for (int64_t q = 0; q < Q; ++q) {
                const int64_t w_ = q * g->sw - g->pw + s;
                if (w_ < 0 || w_ >= g->W) continue;
                acc += (double)dy[YI(n, k, p, q)] * (double)x[XI(n, c, h, w_)];
            }
        }
    return acc;
}

/* dw[k,c,r,s] = sum_{n,p,q} dy[n,k,p,q] * x[n,c,p*sh-ph+r,q*sw-pw+s]. */
void oracle_conv_bwd_weight(const oracle_conv_shape* g, const float* x, const float* dy, double* dw) {
    const int64_t P = oracle_out_extent(g->H, g->R, g->sh, g->ph);
    const int64_t Q = oracle_out_extent(g->W, g->S, g->sw, g->pw);
    const int64_t total = g->K * g->C * g->R * g->S;
    if (P <= 0 || Q <= 0) { memset(dw, 0, sizeof(double) * (size_t)total); return; }
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t i = 0; i < total; ++i) {
        const int64_t s = i % g->S, r = (i / g->S) % g->R;
        const int64_t c = (i / (g->S * g->R)) % g->C, k = i / (g->S * g->R * g->C);
        dw[i] = dw_element(g, x, dy, P, Q, k, c, r, s);
    }
}

/* The same sum for a chosen list of flat dw indices (full-size layers: sampled parity). */
void oracle_conv_bwd_weight_at(const oracle_conv_shape* g, const float* x, const float* dy,
                               const int64_t* flat_idx, int64_t n_idx, double* out) {
    const int64_t P = oracle_out_extent(g->H, g->R, g->sh, g->ph);
    const int64_t Q = oracle_out_extent(g->W, g->S, g->sw, g->pw);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t j = 0; j < n_idx; ++j) {
        const int64_t i = flat_idx[j];
        const int64_t s = i % g->S, r = (i / g->S) % g->R;
        const int64_t c = (i / (g->S * g->R)) % g->C, k = i / (g->S * g->R * g->C);
        out[j] = (P <= 0 || Q <= 0) ? 0.0 : dw_element(g, x, dy, P, Q, k, c, r, s);
    }
}

/* db[k] = sum_{n,p,q} dy[n,k,p,q]. */
void oracle_bias_bwd(const float* dy, double* db, int64_t N, int64_t K, int64_t PQ) {
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < K; ++k) {
        double acc = 0.0;
        for (int64_t n = 0; n < N; ++n) {
            const float* row = dy + (n * K + k) * PQ;
            for (int64_t i = 0; i < PQ; ++i) acc += (double)row[i];
        }
        db[k] = acc;
    }
}

/* ---- exact support operators used to chain layers (not part of the FLOP count) ---- */

/* y = max(x, 0). */
void oracle_relu_fwd(const float* x, float* y, int64_t n) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) y[i] = x[i] > 0.0f ? x[i] : 0.0f;
}

/* dx = dy where x > 0, else 0 (the gradient does not pass at exactly 0). */
void oracle_relu_bwd(const float* x, const float* dy, float* dx, int64_t n) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) dx[i] = x[i] > 0.0f ? dy[i] : 0.0f;
}

/* Max pooling over k x k windows; padded positions never win; the first maximum in row-major
 * window order wins ties. arg holds the flat (h*W + w) position of the winner inside its plane,
 * or -1 for a window that covers no input position. */
void oracle_maxpool_fwd(const float* x, float* y, int32_t* arg, int64_t NC, int64_t H, int64_t W,
                        int64_t k, int64_t stride, int64_t pad) {
    const int64_t P = oracle_out_extent(H, k, stride, pad);
    const int64_t Q = oracle_out_extent(W, k, stride, pad);
    if (P <= 0 || Q <= 0) return;
#pragma omp parallel for schedule(static)
    for (int64_t nc = 0; nc < NC; ++nc)
        for (int64_t p = 0; p < P; ++p)
            for (int64_t q = 0; q < Q; ++q) {
                int32_t best = -1;
                float bv = 0.0f;
                for (int64_t r = 0; r < k; ++r)
                    for (int64_t s = 0; s < k; ++s) {
                        const int64_t h = p * stride - pad + r, w_ = q * stride - pad + s;
                        if (h < 0 || h >= H || w_ < 0 || w_ >= W) continue;
                        const float v = x[(nc * H + h) * W + w_];
                        if (best < 0 || v > bv) { best = (int32_t)(h * W + w_); bv = v; }
                    }
                y[(nc * P + p) * Q + q] = bv;
                arg[(nc * P + p) * Q + q] = best;
            }
}

/* dx[arg] += dy for every window, fp64 accumulation. */
void oracle_maxpool_bwd(const float* dy, const int32_t* arg, double* dx, int64_t NC, int64_t HW,
                        int64_t PQ) {
#pragma omp parallel for schedule(static)
    for (int64_t nc = 0; nc < NC; ++nc) {
        double* plane = dx + nc * HW;
        for (int64_t i = 0; i < HW; ++i) plane[i] = 0.0;
        for (int64_t i = 0; i < PQ; ++i) {
            const int32_t a = arg[nc * PQ + i];
            if (a >= 0) plane[a] += (double)dy[nc * PQ + i];
        }
    }
}

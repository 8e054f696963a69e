/*
 * CPU oracle for the conv + LARS training hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, direct implementations of what one data-parallel worker computes
 * in a training iteration: the convolution forward pass, the two gradients that
 * make up the worker's local gradient ("Data-Parallelism SGD": each worker
 * computes its local gradient independently), and the layer-wise LARS weight
 * update the paper trains with ("Scaling up Batch Size"; hyper-parameters from
 * the AlexNet accuracy table: momentum, weight decay, poly policy of power 2).
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call
 * this.  It shares no code with the HIP library and is not a fallback for it.
 *
 * Arithmetic: every sum is accumulated in double; results are returned as
 * double (convolutions) or rounded once to float (LARS state), so that the
 * only differences to a correct GPU result are summation order and the final
 * rounding.  No blocking, no reordering, no vector intrinsics.  OpenMP is used
 * across independent outputs only (for the timing leg); it never splits a sum.
 *
 * Parity pins (tests/test_oracle_*.py): hand-worked 3x3 example, 1x1 and
 * full-window cases against a matrix product, delta-filter shifts, central
 * finite differences, the adjoint identity, float64 library convolution, and
 * for LARS hand-computed trust ratios and the rule's invariants; for the grouped
 * convolution its reduction to independent convolutions on channel slices, the
 * one-group case, the float64 library convolution and the paper's AlexNet
 * counts.  No function here is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Tensor layouts.  NCHW: activations [N][C][H][W], filter [K][C][R][S] (Caffe blob
 * order, the framework the paper's single-node code is built on).  NHWC:
 * activations [N][H][W][C], filter [K][R][S][C].  Handled by index functions only. */
enum { ORACLE_NCHW = 0, ORACLE_NHWC = 1 };

typedef struct {
    int n, c, h, w;          /* input                          */
    int k, r, s;             /* filter: k outputs, r x s window */
    int stride_h, stride_w, pad_h, pad_w;
    int layout;
} oracle_conv;

static int out_p(const oracle_conv* d) { return (d->h + 2 * d->pad_h - d->r) / d->stride_h + 1; }
static int out_q(const oracle_conv* d) { return (d->w + 2 * d->pad_w - d->s) / d->stride_w + 1; }

static size_t xi(const oracle_conv* d, int n, int c, int h, int w) {
    return d->layout == ORACLE_NHWC ? (((size_t)n * d->h + h) * d->w + w) * d->c + c
                                    : (((size_t)n * d->c + c) * d->h + h) * d->w + w;
}
static size_t wi(const oracle_conv* d, int k, int c, int r, int s) {
    return d->layout == ORACLE_NHWC ? (((size_t)k * d->r + r) * d->s + s) * d->c + c
                                    : (((size_t)k * d->c + c) * d->r + r) * d->s + s;
}
static size_t yi(const oracle_conv* d, int P, int Q, int n, int k, int p, int q) {
    return d->layout == ORACLE_NHWC ? (((size_t)n * P + p) * Q + q) * d->k + k
                                    : (((size_t)n * d->k + k) * P + p) * Q + q;
}

int oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int t) {
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

int oracle_conv2d_out_shape(const oracle_conv* d, int* p, int* q) {
    if (!d || d->n <= 0 || d->c <= 0 || d->h <= 0 || d->w <= 0 || d->k <= 0 || d->r <= 0 || d->s <= 0 ||
        d->stride_h <= 0 || d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0)
        return 1;
    if (d->h + 2 * d->pad_h < d->r || d->w + 2 * d->pad_w < d->s) return 1;
    *p = out_p(d);
    *q = out_q(d);
    return 0;
}

/* Forward: Y[n,k,p,q] = sum_{c,r,s} X[n,c,p*sh-ph+r,q*sw-pw+s] * W[k,c,r,s]; reads outside
 * the image are zero (cross-correlation, no filter flip, floor output size). */
void oracle_conv2d_fwd(const oracle_conv* d, const float* x, const float* wt, double* y) {
    const int P = out_p(d), Q = out_q(d);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < d->n; ++n)
        for (int k = 0; k < d->k; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double acc = 0.0;
                    for (int c = 0; c < d->c; ++c)
                        for (int r = 0; r < d->r; ++r)
                            for (int s = 0; s < d->s; ++s) {
                                const int h = p * d->stride_h - d->pad_h + r;
                                const int w = q * d->stride_w - d->pad_w + s;
                                if (h >= 0 && h < d->h && w >= 0 && w < d->w)
                                    acc += (double)x[xi(d, n, c, h, w)] * (double)wt[wi(d, k, c, r, s)];
                            }
                    y[yi(d, P, Q, n, k, p, q)] = acc;
                }
}

/* Gradient with respect to the input, as the transpose of the forward loop (scatter):
 * every forward term X*W -> Y hands dY*W back to the X element it read. */
void oracle_conv2d_bwd_data(const oracle_conv* d, const float* dy, const float* wt, double* dx) {
    const int P = out_p(d), Q = out_q(d);
    memset(dx, 0, sizeof(double) * (size_t)d->n * d->c * d->h * d->w);
#pragma omp parallel for schedule(static) /* images are independent: each n owns dx[n] */
    for (int n = 0; n < d->n; ++n)
        for (int k = 0; k < d->k; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    const double g = (double)dy[yi(d, P, Q, n, k, p, q)];
                    for (int c = 0; c < d->c; ++c)
                        for (int r = 0; r < d->r; ++r)
                            for (int s = 0; s < d->s; ++s) {
                                const int h = p * d->stride_h - d->pad_h + r;
                                const int w = q * d->stride_w - d->pad_w + s;
                                if (h >= 0 && h < d->h && w >= 0 && w < d->w)
                                    dx[xi(d, n, c, h, w)] += g * (double)wt[wi(d, k, c, r, s)];
                            }
                }
}

/* Gradient with respect to the filter, again as the transposed forward loop. */
void oracle_conv2d_bwd_weight(const oracle_conv* d, const float* x, const float* dy, double* dw) {
    const int P = out_p(d), Q = out_q(d);
    memset(dw, 0, sizeof(double) * (size_t)d->k * d->c * d->r * d->s);
#pragma omp parallel for schedule(static) /* output channels are independent: each k owns dw[k] */
    for (int k = 0; k < d->k; ++k)
        for (int n = 0; n < d->n; ++n)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    const double g = (double)dy[yi(d, P, Q, n, k, p, q)];
                    for (int c = 0; c < d->c; ++c)
                        for (int r = 0; r < d->r; ++r)
                            for (int s = 0; s < d->s; ++s) {
                                const int h = p * d->stride_h - d->pad_h + r;
                                const int w = q * d->stride_w - d->pad_w + s;
                                if (h >= 0 && h < d->h && w >= 0 && w < d->w)
                                    dw[wi(d, k, c, r, s)] += g * (double)x[xi(d, n, c, h, w)];
                            }
                }
}

/* ---- grouped convolution (the original AlexNet of the paper's scaling-ratio table: 61 million parameters and 1.5
 * billion operations per image are the counts of the network whose second, fourth and fifth convolutions are split
 * into two groups).  The c input channels and the k filters are cut into `groups` equal slices; filter k belongs to
 * group k / (k/groups) and sees only that group's c/groups input channels, so the filter tensor is
 * [K][C/groups][R][S] (NHWC: [K][R][S][C/groups]):
 *     Y[n,k,p,q] = sum_{cl < C/groups, r, s} X[n, g(k)*C/groups + cl, p*sh-ph+r, q*sw-pw+s] * W[k,cl,r,s].
 * The two gradients are again the transposed forward loop.  d->c and d->k are the TOTAL channel counts. ---- */
static size_t wgi(const oracle_conv* d, int cg, int k, int cl, int r, int s) {
    return d->layout == ORACLE_NHWC ? (((size_t)k * d->r + r) * d->s + s) * cg + cl
                                    : (((size_t)k * cg + cl) * d->r + r) * d->s + s;
}

void oracle_conv2d_fwd_grouped(const oracle_conv* d, int groups, const float* x, const float* wt, double* y) {
    const int P = out_p(d), Q = out_q(d), cg = d->c / groups, kg = d->k / groups;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < d->n; ++n)
        for (int k = 0; k < d->k; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    const int g = k / kg;
                    double acc = 0.0;
                    for (int cl = 0; cl < cg; ++cl)
                        for (int r = 0; r < d->r; ++r)
                            for (int s = 0; s < d->s; ++s) {
                                const int h = p * d->stride_h - d->pad_h + r;
                                const int w = q * d->stride_w - d->pad_w + s;
                                if (h >= 0 && h < d->h && w >= 0 && w < d->w)
                                    acc += (double)x[xi(d, n, g * cg + cl, h, w)] * (double)wt[wgi(d, cg, k, cl, r, s)];
                            }
                    y[yi(d, P, Q, n, k, p, q)] = acc;
                }
}

void oracle_conv2d_bwd_data_grouped(const oracle_conv* d, int groups, const float* dy, const float* wt, double* dx) {
    const int P = out_p(d), Q = out_q(d), cg = d->c / groups, kg = d->k / groups;
    memset(dx, 0, sizeof(double) * (size_t)d->n * d->c * d->h * d->w);
#pragma omp parallel for schedule(static) /* images are independent: each n owns dx[n] */
    for (int n = 0; n < d->n; ++n)
        for (int k = 0; k < d->k; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    const int g = k / kg;
                    const double gr = (double)dy[yi(d, P, Q, n, k, p, q)];
                    for (int cl = 0; cl < cg; ++cl)
                        for (int r = 0; r < d->r; ++r)
                            for (int s = 0; s < d->s; ++s) {
                                const int h = p * d->stride_h - d->pad_h + r;
                                const int w = q * d->stride_w - d->pad_w + s;
                                if (h >= 0 && h < d->h && w >= 0 && w < d->w)
                                    dx[xi(d, n, g * cg + cl, h, w)] += gr * (double)wt[wgi(d, cg, k, cl, r, s)];
                            }
                }
}

void oracle_conv2d_bwd_weight_grouped(const oracle_conv* d, int groups, const float* x, const float* dy, double* dw) {
    const int P = out_p(d), Q = out_q(d), cg = d->c / groups, kg = d->k / groups;
    memset(dw, 0, sizeof(double) * (size_t)d->k * cg * d->r * d->s);
#pragma omp parallel for schedule(static) /* output channels are independent: each k owns dw[k] */
    for (int k = 0; k < d->k; ++k)
        for (int n = 0; n < d->n; ++n)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    const int g = k / kg;
                    const double gr = (double)dy[yi(d, P, Q, n, k, p, q)];
                    for (int cl = 0; cl < cg; ++cl)
                        for (int r = 0; r < d->r; ++r)
                            for (int s = 0; s < d->s; ++s) {
                                const int h = p * d->stride_h - d->pad_h + r;
                                const int w = q * d->stride_w - d->pad_w + s;
                                if (h >= 0 && h < d->h && w >= 0 && w < d->w)
                                    dw[wgi(d, cg, k, cl, r, s)] += gr * (double)x[xi(d, n, g * cg + cl, h, w)];
                            }
                }
}

/* ---- single output elements (gather form), for sampled checks at full benchmark sizes.
 * coords is [count][4] int32.  abs_out (may be NULL) receives sum |term|, the scale against
 * which a summation-order error is bounded. ---- */

void oracle_conv2d_fwd_at(const oracle_conv* d, const float* x, const float* wt, const int32_t* coords,
                          int64_t count, double* out, double* abs_out) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        const int n = coords[4 * i], k = coords[4 * i + 1], p = coords[4 * i + 2], q = coords[4 * i + 3];
        double acc = 0.0, mag = 0.0;
        for (int c = 0; c < d->c; ++c)
            for (int r = 0; r < d->r; ++r)
                for (int s = 0; s < d->s; ++s) {
                    const int h = p * d->stride_h - d->pad_h + r;
                    const int w = q * d->stride_w - d->pad_w + s;
                    if (h >= 0 && h < d->h && w >= 0 && w < d->w) {
                        const double t = (double)x[xi(d, n, c, h, w)] * (double)wt[wi(d, k, c, r, s)];
                        acc += t;
                        mag += fabs(t);
                    }
                }
        out[i] = acc;
        if (abs_out) abs_out[i] = mag;
    }
}

/* dX[n,c,h,w]: sum over the (k,p,q,r,s) whose forward read hit (h,w). */
void oracle_conv2d_bwd_data_at(const oracle_conv* d, const float* dy, const float* wt, const int32_t* coords,
                               int64_t count, double* out, double* abs_out) {
    const int P = out_p(d), Q = out_q(d);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        const int n = coords[4 * i], c = coords[4 * i + 1], h = coords[4 * i + 2], w = coords[4 * i + 3];
        double acc = 0.0, mag = 0.0;
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q) {
                const int r = h - (p * d->stride_h - d->pad_h);
                const int s = w - (q * d->stride_w - d->pad_w);
                if (r < 0 || r >= d->r || s < 0 || s >= d->s) continue;
                for (int k = 0; k < d->k; ++k) {
                    const double t = (double)dy[yi(d, P, Q, n, k, p, q)] * (double)wt[wi(d, k, c, r, s)];
                    acc += t;
                    mag += fabs(t);
                }
            }
        out[i] = acc;
        if (abs_out) abs_out[i] = mag;
    }
}

/* dW[k,c,r,s]: sum over the batch and all output positions. */
void oracle_conv2d_bwd_weight_at(const oracle_conv* d, const float* x, const float* dy, const int32_t* coords,
                                 int64_t count, double* out, double* abs_out) {
    const int P = out_p(d), Q = out_q(d);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        const int k = coords[4 * i], c = coords[4 * i + 1], r = coords[4 * i + 2], s = coords[4 * i + 3];
        double acc = 0.0, mag = 0.0;
        for (int n = 0; n < d->n; ++n)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    const int h = p * d->stride_h - d->pad_h + r;
                    const int w = q * d->stride_w - d->pad_w + s;
                    if (h >= 0 && h < d->h && w >= 0 && w < d->w) {
                        const double t = (double)dy[yi(d, P, Q, n, k, p, q)] * (double)x[xi(d, n, c, h, w)];
                        acc += t;
                        mag += fabs(t);
                    }
                }
        out[i] = acc;
        if (abs_out) abs_out[i] = mag;
    }
}

/* ---- LARS ----
 * The paper names the rule and cites it; it is the layer-wise rule of the LARS paper it
 * builds on.  Per tensor ("layer") l, with trust coefficient eta, weight decay beta,
 * momentum m and global rate gamma (set by the poly schedule below):
 *     lambda_l = eta * ||w_l|| / (||g_l|| + beta * ||w_l||)        (Euclidean norms of raw w, g)
 *     v_l <- m * v_l + gamma * lambda_l * (g_l + beta * w_l)
 *     w_l <- w_l - v_l
 * Where the quotient is undefined (||w_l|| = 0, or the denominator is 0) lambda_l = 1.
 * w and v are updated in place (stored as float); norms_out (may be NULL) receives
 * ||w||, ||g|| per tensor and trust_out (may be NULL) lambda per tensor, in double. */
void oracle_lars_step(int n_tensors, float* const* w, const float* const* g, float* const* v,
                      const int64_t* numel, double eta, double momentum, double weight_decay, double lr,
                      double* trust_out, double* norms_out) {
#pragma omp parallel for schedule(dynamic, 1) /* tensors are independent */
    for (int l = 0; l < n_tensors; ++l) {
        double sw = 0.0, sg = 0.0;
        for (int64_t i = 0; i < numel[l]; ++i) {
            sw += (double)w[l][i] * (double)w[l][i];
            sg += (double)g[l][i] * (double)g[l][i];
        }
        const double nw = sqrt(sw), ng = sqrt(sg);
        const double den = ng + weight_decay * nw;
        const double lambda = (nw > 0.0 && den > 0.0) ? eta * nw / den : 1.0;
        for (int64_t i = 0; i < numel[l]; ++i) {
            const double vi = momentum * (double)v[l][i] + lr * lambda * ((double)g[l][i] + weight_decay * (double)w[l][i]);
            v[l][i] = (float)vi;
            w[l][i] = (float)((double)w[l][i] - vi);
        }
        if (trust_out) trust_out[l] = lambda;
        if (norms_out) {
            norms_out[2 * l] = nw;
            norms_out[2 * l + 1] = ng;
        }
    }
}

/* The same rule with per-tensor coefficients.  The paper applies the rule layer by layer ("Layer-wise
 * Adaptive Rate Scaling", "Scaling up Batch Size"); which tensors take part, and with which eta and
 * beta, is left to the user of the rule -- biases and batch-norm parameters are commonly given no
 * layer-wise scaling.  eta_l and beta_l override the scalars where the arrays are not NULL; a tensor
 * with skip[l] != 0 takes lambda_l = 1 (plain momentum SGD with its weight decay). */
void oracle_lars_step_ex(int n_tensors, float* const* w, const float* const* g, float* const* v,
                         const int64_t* numel, double eta, double momentum, double weight_decay, double lr,
                         const double* eta_l, const double* beta_l, const unsigned char* skip,
                         double* trust_out, double* norms_out) {
#pragma omp parallel for schedule(dynamic, 1) /* tensors are independent */
    for (int l = 0; l < n_tensors; ++l) {
        const double eta_here = eta_l ? eta_l[l] : eta;
        const double beta = beta_l ? beta_l[l] : weight_decay;
        double sw = 0.0, sg = 0.0;
        for (int64_t i = 0; i < numel[l]; ++i) {
            sw += (double)w[l][i] * (double)w[l][i];
            sg += (double)g[l][i] * (double)g[l][i];
        }
        const double nw = sqrt(sw), ng = sqrt(sg);
        const double den = ng + beta * nw;
        double lambda = (nw > 0.0 && den > 0.0) ? eta_here * nw / den : 1.0;
        if (skip && skip[l]) lambda = 1.0;
        for (int64_t i = 0; i < numel[l]; ++i) {
            const double vi = momentum * (double)v[l][i] + lr * lambda * ((double)g[l][i] + beta * (double)w[l][i]);
            v[l][i] = (float)vi;
            w[l][i] = (float)((double)w[l][i] - vi);
        }
        if (trust_out) trust_out[l] = lambda;
        if (norms_out) {
            norms_out[2 * l] = nw;
            norms_out[2 * l + 1] = ng;
        }
    }
}

/* Warm-up followed by the poly policy.  The paper's warm-up scheme starts from a small rate and raises it to
 * the large one over the first few epochs ("Difficulty of Large-Batch Training"; 5 epochs for ResNet-50);
 * the shape of the ramp is not printed and is taken to be linear.  For t < W:
 *     gamma_t = gamma_start + (gamma_0 - gamma_start) * t / W
 * and from t = W on the poly policy runs over the remaining T - W iterations, starting at gamma_0:
 *     gamma_t = gamma_0 * (1 - (t - W)/(T - W))^power. */
double oracle_warmup_poly_lr(double base_lr, double start_lr, int64_t iter, int64_t warmup_iters, int64_t max_iter,
                             double power) {
    if (warmup_iters > 0 && iter < warmup_iters)
        return start_lr + (base_lr - start_lr) * (double)iter / (double)warmup_iters;
    const int64_t w = warmup_iters > 0 ? warmup_iters : 0;
    if (max_iter <= w) return base_lr;
    double frac = 1.0 - (double)(iter - w) / (double)(max_iter - w);
    if (frac < 0.0) frac = 0.0;
    return base_lr * pow(frac, power);
}

/* Poly learning-rate policy: gamma_t = gamma_0 * (1 - t/T)^power; the paper uses power 2. */
double oracle_poly_lr(double base_lr, int64_t iter, int64_t max_iter, double power) {
    if (max_iter <= 0) return base_lr;
    double frac = 1.0 - (double)iter / (double)max_iter;
    if (frac < 0.0) frac = 0.0;
    return base_lr * pow(frac, power);
}

/*
 * CPU oracle for the batched-lowering convolution path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition of what the GPU library must compute.  It is
 * written from the paper (Omnivore, arXiv 1606.04487) and shares no code, header, table
 * or helper with the HIP sources; only tests, the smoke check and the bench's CPU-baseline
 * leg may call it.  All accumulation is in double precision; inputs are float arrays whose
 * values are used exactly (a bf16 value is a float, so the same entry points serve both
 * storage types).
 *
 * What follows which passage:
 *   forward ............ Sec. III-A, Eq. (conv_full) and its restatement in App. C
 *                        ("Convolutional Layer Computation"): a sum over input channels and
 *                        the k x k window of data times kernel, with no kernel flip.  Stride
 *                        and zero padding are the two parameters App. C says the kernel
 *                        "also supports"; the equation is the case stride 1, pad k/2 and
 *                        App. C's m = n-k+1 is the case stride 1, pad 0.
 *   backward ........... Sec. II-B: the BW operation takes the gradient w.r.t. the layer's
 *                        output and returns the gradient w.r.t. its input, and computes the
 *                        gradient w.r.t. the model; gradients of the images of a batch are
 *                        summed (no 1/b).  Both are the adjoints of the forward sum, written
 *                        here as the same seven loops with a different accumulation target.
 *   lowering / lifting . App. C "Convolution by Lowering and GEMM": D-hat holds replicated
 *                        data so that the layer becomes one matrix product; D-hat is the
 *                        "B" operand whose columns grow with the number of images.
 *   update ............. Sec. II-B, Eq. (update1), (update2).
 *   ReLU / max-pool .... named only (App. C, "Data Parallelism in non-GEMM Kernels"); the
 *                        tie and border rules are this build's readings.
 *   normalisation, dropout  named in the same passage; formulas and the random generator are
 *                        readings stated above the routines.
 *
 * Layouts: X [N][C][H][W], Wt [F][C][kh][kw], Y [N][F][Ho][Wo], all contiguous.
 * D-hat is row-major [C*kh*kw][N*Ho*Wo]: row (c*kh+ky)*kw+kx, column (n*Ho+oy)*Wo+ox.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t N, C, H, W;      /* input batch, channels, height, width */
    int32_t F, kh, kw;       /* filters, window */
    int32_t sh, sw, ph, pw;  /* stride, zero padding */
} oc_shape;

/* Threads the parallel loops below will use. */
int oc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Output extent: number of window positions that fit entirely inside the padded input. */
int oc_out_dims(const oc_shape *s, int32_t *Ho, int32_t *Wo)
{
    if (s->N <= 0 || s->C <= 0 || s->H <= 0 || s->W <= 0 || s->F <= 0 || s->kh <= 0 ||
        s->kw <= 0 || s->sh <= 0 || s->sw <= 0 || s->ph < 0 || s->pw < 0)
        return -1;
    int64_t eh = (int64_t)s->H + 2 * s->ph - s->kh;
    int64_t ew = (int64_t)s->W + 2 * s->pw - s->kw;
    if (eh < 0 || ew < 0)
        return -1;
    *Ho = (int32_t)(eh / s->sh) + 1;
    *Wo = (int32_t)(ew / s->sw) + 1;
    return 0;
}

#define XI(n, c, y, x) ((((int64_t)(n) * s->C + (c)) * s->H + (y)) * s->W + (x))
#define WI(f, c, ky, kx) ((((int64_t)(f) * s->C + (c)) * s->kh + (ky)) * s->kw + (kx))
#define YI(n, f, oy, ox) ((((int64_t)(n) * s->F + (f)) * Ho + (oy)) * Wo + (ox))

/* Forward, Eq. (conv_full) with stride and padding: seven loops n, f, oy, ox, c, ky, kx. */
void oc_conv_forward(const oc_shape *s, const float *X, const float *Wt, const float *bias,
                     double *Y)
{
    int32_t Ho, Wo;
    if (oc_out_dims(s, &Ho, &Wo))
        return;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < s->N; ++n)
        for (int f = 0; f < s->F; ++f)
            for (int oy = 0; oy < Ho; ++oy)
                for (int ox = 0; ox < Wo; ++ox) {
                    double acc = 0.0;
                    for (int c = 0; c < s->C; ++c)
                        for (int ky = 0; ky < s->kh; ++ky)
                            for (int kx = 0; kx < s->kw; ++kx) {
                                int iy = oy * s->sh - s->ph + ky;
                                int ix = ox * s->sw - s->pw + kx;
                                if (iy < 0 || iy >= s->H || ix < 0 || ix >= s->W)
                                    continue; /* zero padding */
                                acc += (double)X[XI(n, c, iy, ix)] * (double)Wt[WI(f, c, ky, kx)];
                            }
                    if (bias)
                        acc += (double)bias[f];
                    Y[YI(n, f, oy, ox)] = acc;
                }
}

/* Data gradient: the forward loops, accumulating into dX instead of Y (scatter form). */
void oc_conv_backward_data(const oc_shape *s, const float *dY, const float *Wt, double *dX)
{
    int32_t Ho, Wo;
    if (oc_out_dims(s, &Ho, &Wo))
        return;
    memset(dX, 0, sizeof(double) * (size_t)s->N * s->C * s->H * s->W);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < s->N; ++n) /* images write disjoint parts of dX */
        for (int f = 0; f < s->F; ++f)
            for (int oy = 0; oy < Ho; ++oy)
                for (int ox = 0; ox < Wo; ++ox) {
                    double g = (double)dY[YI(n, f, oy, ox)];
                    for (int c = 0; c < s->C; ++c)
                        for (int ky = 0; ky < s->kh; ++ky)
                            for (int kx = 0; kx < s->kw; ++kx) {
                                int iy = oy * s->sh - s->ph + ky;
                                int ix = ox * s->sw - s->pw + kx;
                                if (iy < 0 || iy >= s->H || ix < 0 || ix >= s->W)
                                    continue;
                                dX[XI(n, c, iy, ix)] += g * (double)Wt[WI(f, c, ky, kx)];
                            }
                }
}

/* Model gradient, summed over the batch: the forward loops, accumulating into dW. */
void oc_conv_backward_weights(const oc_shape *s, const float *X, const float *dY, double *dW)
{
    int32_t Ho, Wo;
    if (oc_out_dims(s, &Ho, &Wo))
        return;
    memset(dW, 0, sizeof(double) * (size_t)s->F * s->C * s->kh * s->kw);
#pragma omp parallel for schedule(static)
    for (int f = 0; f < s->F; ++f) /* filters write disjoint parts of dW */
        for (int n = 0; n < s->N; ++n)
            for (int oy = 0; oy < Ho; ++oy)
                for (int ox = 0; ox < Wo; ++ox) {
                    double g = (double)dY[YI(n, f, oy, ox)];
                    for (int c = 0; c < s->C; ++c)
                        for (int ky = 0; ky < s->kh; ++ky)
                            for (int kx = 0; kx < s->kw; ++kx) {
                                int iy = oy * s->sh - s->ph + ky;
                                int ix = ox * s->sw - s->pw + kx;
                                if (iy < 0 || iy >= s->H || ix < 0 || ix >= s->W)
                                    continue;
                                dW[WI(f, c, ky, kx)] += g * (double)X[XI(n, c, iy, ix)];
                            }
                }
}

/* Bias gradient: plain sum of the upstream gradient over images and output pixels. */
void oc_bias_grad(const oc_shape *s, const float *dY, double *dbias)
{
    int32_t Ho, Wo;
    if (oc_out_dims(s, &Ho, &Wo))
        return;
    for (int f = 0; f < s->F; ++f) {
        double acc = 0.0;
        for (int n = 0; n < s->N; ++n)
            for (int oy = 0; oy < Ho; ++oy)
                for (int ox = 0; ox < Wo; ++ox)
                    acc += (double)dY[YI(n, f, oy, ox)];
        dbias[f] = acc;
    }
}

/*
 * Single entries, for parity at sizes where the full loops would take hours.  Each takes a
 * list of flat indices into the result tensor and evaluates only those entries.
 */
void oc_conv_forward_at(const oc_shape *s, const float *X, const float *Wt, const float *bias,
                        const int64_t *idx, int64_t count, double *out)
{
    int32_t Ho, Wo;
    if (oc_out_dims(s, &Ho, &Wo))
        return;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t q = 0; q < count; ++q) {
        int64_t t = idx[q];
        int ox = (int)(t % Wo); t /= Wo;
        int oy = (int)(t % Ho); t /= Ho;
        int f = (int)(t % s->F);
        int n = (int)(t / s->F);
        double acc = 0.0;
        for (int c = 0; c < s->C; ++c)
            for (int ky = 0; ky < s->kh; ++ky)
                for (int kx = 0; kx < s->kw; ++kx) {
                    int iy = oy * s->sh - s->ph + ky;
                    int ix = ox * s->sw - s->pw + kx;
                    if (iy < 0 || iy >= s->H || ix < 0 || ix >= s->W)
                        continue;
                    acc += (double)X[XI(n, c, iy, ix)] * (double)Wt[WI(f, c, ky, kx)];
                }
        if (bias)
            acc += (double)bias[f];
        out[q] = acc;
    }
}

/* One dX entry (gather form): every (f, ky, kx) whose window position lands on (iy, ix). */
void oc_conv_backward_data_at(const oc_shape *s, const float *dY, const float *Wt,
                              const int64_t *idx, int64_t count, double *out)
{
    int32_t Ho, Wo;
    if (oc_out_dims(s, &Ho, &Wo))
        return;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t q = 0; q < count; ++q) {
        int64_t t = idx[q];
        int ix = (int)(t % s->W); t /= s->W;
        int iy = (int)(t % s->H); t /= s->H;
        int c = (int)(t % s->C);
        int n = (int)(t / s->C);
        double acc = 0.0;
        for (int f = 0; f < s->F; ++f)
            for (int ky = 0; ky < s->kh; ++ky)
                for (int kx = 0; kx < s->kw; ++kx) {
                    int ty = iy + s->ph - ky, tx = ix + s->pw - kx;
                    if (ty < 0 || tx < 0 || ty % s->sh || tx % s->sw)
                        continue;
                    int oy = ty / s->sh, ox = tx / s->sw;
                    if (oy >= Ho || ox >= Wo)
                        continue;
                    acc += (double)dY[YI(n, f, oy, ox)] * (double)Wt[WI(f, c, ky, kx)];
                }
        out[q] = acc;
    }
}

/* One dW entry: sum over every image and output pixel. */
void oc_conv_backward_weights_at(const oc_shape *s, const float *X, const float *dY,
                                 const int64_t *idx, int64_t count, double *out)
{
    int32_t Ho, Wo;
    if (oc_out_dims(s, &Ho, &Wo))
        return;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t q = 0; q < count; ++q) {
        int64_t t = idx[q];
        int kx = (int)(t % s->kw); t /= s->kw;
        int ky = (int)(t % s->kh); t /= s->kh;
        int c = (int)(t % s->C);
        int f = (int)(t / s->C);
        double acc = 0.0;
        for (int n = 0; n < s->N; ++n)
            for (int oy = 0; oy < Ho; ++oy)
                for (int ox = 0; ox < Wo; ++ox) {
                    int iy = oy * s->sh - s->ph + ky;
                    int ix = ox * s->sw - s->pw + kx;
                    if (iy < 0 || iy >= s->H || ix < 0 || ix >= s->W)
                        continue;
                    acc += (double)dY[YI(n, f, oy, ox)] * (double)X[XI(n, c, iy, ix)];
                }
        out[q] = acc;
    }
}

/*
 * Lowering: D-hat[(c,ky,kx)][(n,oy,ox)] = X[n,c,oy*sh-ph+ky,ox*sw-pw+kx], or +0 in the padding.
 * A pure copy: every entry is a bit pattern of X or zero.
 */
void oc_lower(const oc_shape *s, const float *X, float *Dhat)
{
    int32_t Ho, Wo;
    if (oc_out_dims(s, &Ho, &Wo))
        return;
    int64_t M = (int64_t)s->N * Ho * Wo;
#pragma omp parallel for collapse(2) schedule(static)
    for (int c = 0; c < s->C; ++c)
        for (int ky = 0; ky < s->kh; ++ky)
            for (int kx = 0; kx < s->kw; ++kx) {
                int64_t row = ((int64_t)c * s->kh + ky) * s->kw + kx;
                for (int n = 0; n < s->N; ++n)
                    for (int oy = 0; oy < Ho; ++oy)
                        for (int ox = 0; ox < Wo; ++ox) {
                            int iy = oy * s->sh - s->ph + ky;
                            int ix = ox * s->sw - s->pw + kx;
                            int64_t col = ((int64_t)n * Ho + oy) * Wo + ox;
                            float v = 0.0f;
                            if (iy >= 0 && iy < s->H && ix >= 0 && ix < s->W)
                                v = X[XI(n, c, iy, ix)];
                            Dhat[row * M + col] = v;
                        }
            }
}

/* col2im: the transpose of the 0/1 lowering map; every D-hat-shaped entry is added to the
 * one input position it was copied from (entries that sit in the padding are dropped). */
void oc_col2im(const oc_shape *s, const float *dDhat, double *dX)
{
    int32_t Ho, Wo;
    if (oc_out_dims(s, &Ho, &Wo))
        return;
    int64_t M = (int64_t)s->N * Ho * Wo;
    memset(dX, 0, sizeof(double) * (size_t)s->N * s->C * s->H * s->W);
#pragma omp parallel for schedule(static)
    for (int c = 0; c < s->C; ++c) /* channels write disjoint parts of dX */
        for (int ky = 0; ky < s->kh; ++ky)
            for (int kx = 0; kx < s->kw; ++kx) {
                int64_t row = ((int64_t)c * s->kh + ky) * s->kw + kx;
                for (int n = 0; n < s->N; ++n)
                    for (int oy = 0; oy < Ho; ++oy)
                        for (int ox = 0; ox < Wo; ++ox) {
                            int iy = oy * s->sh - s->ph + ky;
                            int ix = ox * s->sw - s->pw + kx;
                            if (iy < 0 || iy >= s->H || ix < 0 || ix >= s->W)
                                continue;
                            int64_t col = ((int64_t)n * Ho + oy) * Wo + ox;
                            dX[XI(n, c, iy, ix)] += (double)dDhat[row * M + col];
                        }
            }
}

/* Plain triple-loop matrix product in double: C[m][n] = sum_k A[m][k] * B[k][n]. */
void oc_matmul(int64_t m, int64_t k, int64_t n, const double *A, const double *B, double *C)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < n; ++j) {
            double acc = 0.0;
            for (int64_t p = 0; p < k; ++p)
                acc += A[i * k + p] * B[p * n + j];
            C[i * n + j] = acc;
        }
}

/* ReLU: max(0, x); its gradient passes where the input was strictly positive. */
void oc_relu_forward(int64_t count, const float *x, double *y)
{
    for (int64_t i = 0; i < count; ++i)
        y[i] = x[i] > 0.0f ? (double)x[i] : 0.0;
}

void oc_relu_backward(int64_t count, const float *x, const float *dy, double *dx)
{
    for (int64_t i = 0; i < count; ++i)
        dx[i] = x[i] > 0.0f ? (double)dy[i] : 0.0;
}

/* Pooled extent without padding.  ceil_mode keeps a last, border-clipped window. */
int oc_pool_out_dim(int32_t in, int32_t k, int32_t stride, int32_t ceil_mode)
{
    if (in < k || k <= 0 || stride <= 0)
        return -1;
    int32_t span = in - k;
    int32_t o = (ceil_mode ? (span + stride - 1) / stride : span / stride) + 1;
    return o;
}

/* Max-pool over `planes` independent H x W planes.  The first maximum in (ky, kx) scan order
 * wins; argmax is its flat position iy*W+ix inside the plane. */
void oc_maxpool_forward(int64_t planes, int32_t H, int32_t W, int32_t k, int32_t stride,
                        int32_t ceil_mode, const float *x, double *y, int32_t *argmax)
{
    int Ho = oc_pool_out_dim(H, k, stride, ceil_mode);
    int Wo = oc_pool_out_dim(W, k, stride, ceil_mode);
    if (Ho < 0 || Wo < 0)
        return;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < planes; ++p)
        for (int oy = 0; oy < Ho; ++oy)
            for (int ox = 0; ox < Wo; ++ox) {
                int best = -1;
                float bv = 0.0f;
                for (int ky = 0; ky < k; ++ky)
                    for (int kx = 0; kx < k; ++kx) {
                        int iy = oy * stride + ky, ix = ox * stride + kx;
                        if (iy >= H || ix >= W)
                            continue; /* window clipped at the border */
                        float v = x[(p * H + iy) * W + ix];
                        if (best < 0 || v > bv) {
                            best = iy * W + ix;
                            bv = v;
                        }
                    }
                y[(p * Ho + oy) * Wo + ox] = (double)bv;
                argmax[(p * Ho + oy) * Wo + ox] = best;
            }
}

/* Max-pool backward: each pooled gradient goes to the position that won its window. */
void oc_maxpool_backward(int64_t planes, int32_t H, int32_t W, int32_t Ho, int32_t Wo,
                         const float *dy, const int32_t *argmax, double *dx)
{
    memset(dx, 0, sizeof(double) * (size_t)planes * H * W);
    for (int64_t p = 0; p < planes; ++p)
        for (int64_t o = 0; o < (int64_t)Ho * Wo; ++o)
            dx[p * H * W + argmax[p * Ho * Wo + o]] += (double)dy[p * Ho * Wo + o];
}

/* Momentum SGD, Eq. (update2) then Eq. (update1): the step from the old model, then the add. */
void oc_sgd_momentum(int64_t count, const float *W0, const float *V0, const float *G, double lr,
                     double mu, double lambda, double *W1, double *V1)
{
    for (int64_t i = 0; i < count; ++i) {
        double v = mu * (double)V0[i] - lr * ((double)G[i] + lambda * (double)W0[i]);
        V1[i] = v;
        W1[i] = (double)W0[i] + v;
    }
}

/*
 * Local response normalisation across channels and dropout: the two remaining non-GEMM layers
 * of the paper's CaffeNet runs (App. C, "Data Parallelism in non-GEMM Kernels" names them
 * next to pooling and ReLU; the paper gives no formula).  Reading: the normalisation of the
 * AlexNet network the paper trains, in the convention of the framework whose outputs the paper
 * matches layer by layer (the window sum is scaled by alpha / size, and channels beyond the
 * ends count as zero):
 *     s[n,c,p] = k + (alpha / size) * sum_{|c' - c| <= (size-1)/2, 0 <= c' < C} x[n,c',p]^2     (size odd)
 *     y[n,c,p] = x[n,c,p] * s[n,c,p]^(-beta)
 * and its gradient
 *     dx[n,c,p] = dy[n,c,p] * s[n,c,p]^(-beta)
 *                 - (2 alpha beta / size) * x[n,c,p] * sum_{c' : c in window(c')} dy[n,c',p] * x[n,c',p] * s[n,c',p]^(-beta-1)
 * x is [N][C][plane].
 */
static double lrn_scale(const float *x, int64_t C, int64_t plane, int64_t n, int64_t c, int64_t p,
                        int32_t size, double alpha, double k)
{
    double acc = 0.0;
    int64_t lo = c - (size - 1) / 2, hi = c + (size - 1) / 2;  /* size is odd */
    for (int64_t cc = lo; cc <= hi; ++cc) {
        if (cc < 0 || cc >= C)
            continue;
        double v = (double)x[(n * C + cc) * plane + p];
        acc += v * v;
    }
    return k + alpha / (double)size * acc;
}

void oc_lrn_forward(int64_t N, int64_t C, int64_t plane, int32_t size, double alpha, double beta,
                    double k, const float *x, double *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t c = 0; c < C; ++c)
            for (int64_t p = 0; p < plane; ++p) {
                double s = lrn_scale(x, C, plane, n, c, p, size, alpha, k);
                y[(n * C + c) * plane + p] = (double)x[(n * C + c) * plane + p] * pow(s, -beta);
            }
}

void oc_lrn_backward(int64_t N, int64_t C, int64_t plane, int32_t size, double alpha, double beta,
                     double k, const float *x, const float *dy, double *dx)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t c = 0; c < C; ++c)
            for (int64_t p = 0; p < plane; ++p) {
                double xc = (double)x[(n * C + c) * plane + p];
                double own = (double)dy[(n * C + c) * plane + p] *
                             pow(lrn_scale(x, C, plane, n, c, p, size, alpha, k), -beta);
                /* channels c' whose window contains c: the window is symmetric, so |c' - c| <= (size-1)/2 */
                double cross = 0.0;
                for (int64_t cc = c - (size - 1) / 2; cc <= c + (size - 1) / 2; ++cc) {
                    if (cc < 0 || cc >= C)
                        continue;
                    double s = lrn_scale(x, C, plane, n, cc, p, size, alpha, k);
                    cross += (double)dy[(n * C + cc) * plane + p] * (double)x[(n * C + cc) * plane + p] *
                             pow(s, -beta - 1.0);
                }
                dx[(n * C + c) * plane + p] = own - 2.0 * alpha * beta / (double)size * xc * cross;
            }
}

/*
 * Dropout (training mode, as the framework the paper matches applies it): every element is
 * kept with probability 1 - p and scaled by 1 / (1 - p), otherwise set to zero; the backward
 * pass applies the same mask and scale to the gradient.  The random bits come from the
 * counter-based generator Philox4x64-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers:
 * as easy as 1, 2, 3", SC'11): block b = philox(counter = {b, 0, 0, 0}, key = {seed, stream})
 * gives four 64-bit words = eight 32-bit draws (low half first); element i takes draw i mod 8 of
 * block i / 8 and is kept iff draw >= threshold, threshold = floor(p * 2^32) (at most 2^32 - 1).
 */
static void mulhilo64(uint64_t a, uint64_t b, uint64_t *hi, uint64_t *lo)
{
    unsigned __int128 p = (unsigned __int128)a * (unsigned __int128)b;
    *hi = (uint64_t)(p >> 64);
    *lo = (uint64_t)p;
}

void oc_philox4x64(const uint64_t ctr[4], const uint64_t key[2], uint64_t out[4])
{
    const uint64_t M0 = 0xD2E7470EE14C6C93ull, M1 = 0xCA5A826395121157ull;   /* round multipliers */
    const uint64_t W0 = 0x9E3779B97F4A7C15ull, W1 = 0xBB67AE8584CAA73Bull;   /* key increments */
    uint64_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        uint64_t hi0, lo0, hi1, lo1;
        mulhilo64(M0, c0, &hi0, &lo0);
        mulhilo64(M1, c2, &hi1, &lo1);
        uint64_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0, c1 = lo1, c2 = n2, c3 = lo0;
        k0 += W0, k1 += W1;
    }
    out[0] = c0, out[1] = c1, out[2] = c2, out[3] = c3;
}

uint32_t oc_dropout_threshold(double p)
{
    double t = floor(p * 4294967296.0);
    if (t < 0.0)
        t = 0.0;
    if (t > 4294967295.0)
        t = 4294967295.0;
    return (uint32_t)t;
}

/* keep[i] = 1 iff element i survives */
void oc_dropout_mask(int64_t count, double p, uint64_t seed, uint64_t stream, uint8_t *keep)
{
    uint32_t thr = oc_dropout_threshold(p);
    uint64_t key[2] = {seed, stream};
    for (int64_t b = 0; b * 8 < count; ++b) {
        uint64_t ctr[4] = {(uint64_t)b, 0, 0, 0}, w[4];
        oc_philox4x64(ctr, key, w);
        for (int j = 0; j < 8 && b * 8 + j < count; ++j) {
            uint32_t draw = (uint32_t)(j & 1 ? w[j >> 1] >> 32 : w[j >> 1] & 0xffffffffull);
            keep[b * 8 + j] = draw >= thr ? 1 : 0;
        }
    }
}

/* y = keep ? x / (1 - p) : 0.  The same routine maps dy to dx in the backward pass. */
void oc_dropout_apply(int64_t count, double p, uint64_t seed, uint64_t stream, const float *x, double *y)
{
    uint32_t thr = oc_dropout_threshold(p);
    uint64_t key[2] = {seed, stream};
    double scale = 1.0 / (1.0 - p);
    for (int64_t b = 0; b * 8 < count; ++b) {
        uint64_t ctr[4] = {(uint64_t)b, 0, 0, 0}, w[4];
        oc_philox4x64(ctr, key, w);
        for (int j = 0; j < 8 && b * 8 + j < count; ++j) {
            uint32_t draw = (uint32_t)(j & 1 ? w[j >> 1] >> 32 : w[j >> 1] & 0xffffffffull);
            y[b * 8 + j] = draw >= thr ? (double)x[b * 8 + j] * scale : 0.0;
        }
    }
}

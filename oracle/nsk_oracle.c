/*
 * CPU oracle for the residual-CNN training hot path: 2-D convolution forward,
 * backward-data, backward-weight, batch-norm + ReLU + residual-add forward and
 * backward, and 3x3-style max pooling.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the plain definition of every operation,
 * written as direct nested loops in fp64, and is deliberately slow.  Only the
 * tests, the smoke check and the bench's cpu_baseline leg may call it; the
 * product path never does.  It shares no code with the GPU library.
 *
 * Where the operations come from.  The paper hands convolutions to a vendor
 * library (abstract; section "Experiments and Discussion") and trains residual
 * networks "by the ResNet recipe" (same section) without printing formulas, so
 * the definitions here are the textbook ones that recipe implies:
 *   - convolution is cross-correlation with zero padding (no filter flip);
 *   - batch-norm uses batch statistics with the biased variance;
 *   - the gradient of an addition is forwarded unchanged to both operands and
 *     gradients are accumulated into buffers that already hold a value
 *     (section "Automatic Differentiation", the y = x@w + x example; section
 *     "Caching and Pooling" for weight gradients).
 *
 * Layouts: activations NCHW, filters KCRS, everything double, C-contiguous.
 * dims = {N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w}.
 * Threading: one OpenMP "parallel for" over the outermost independent loop.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int N, C, H, W, K, R, S, sh, sw, ph, pw, dh, dw;
} conv_dims;

static int out_extent(int in, int pad, int dil, int filt, int stride)
{
    int span = in + 2 * pad - dil * (filt - 1) - 1;
    return span < 0 ? 0 : span / stride + 1;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_conv2d_out_dims(const int32_t *dims, int32_t *P, int32_t *Q)
{
    const conv_dims *d = (const conv_dims *)dims;
    *P = out_extent(d->H, d->ph, d->dh, d->R, d->sh);
    *Q = out_extent(d->W, d->pw, d->dw, d->S, d->sw);
}

/* y[n,k,p,q] = sum_{c,r,s} x[n,c,p*sh-ph+r*dh,q*sw-pw+s*dw] * w[k,c,r,s],
 * input positions outside the image count as zero. */
void oracle_conv2d_fwd(const double *x, const double *w, double *y, const int32_t *dims)
{
    const conv_dims d = *(const conv_dims *)dims;
    const int P = out_extent(d.H, d.ph, d.dh, d.R, d.sh);
    const int Q = out_extent(d.W, d.pw, d.dw, d.S, d.sw);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < d.N; ++n)
        for (int k = 0; k < d.K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double acc = 0.0;
                    for (int c = 0; c < d.C; ++c)
                        for (int r = 0; r < d.R; ++r) {
                            const int h = p * d.sh - d.ph + r * d.dh;
                            if (h < 0 || h >= d.H) continue;
                            for (int s = 0; s < d.S; ++s) {
                                const int v = q * d.sw - d.pw + s * d.dw;
                                if (v < 0 || v >= d.W) continue;
                                acc += x[(((size_t)n * d.C + c) * d.H + h) * d.W + v] *
                                       w[(((size_t)k * d.C + c) * d.R + r) * d.S + s];
                            }
                        }
                    y[(((size_t)n * d.K + k) * P + p) * Q + q] = acc;
                }
}

/* Adjoint of the forward map with respect to x, written as a scatter: every
 * product the forward pass formed sends dy*w back to the x element it read.
 * accumulate = 0 starts from zero, 1 adds to what dx already holds. */
void oracle_conv2d_dgrad(const double *dy, const double *w, double *dx, const int32_t *dims,
                         int accumulate)
{
    const conv_dims d = *(const conv_dims *)dims;
    const int P = out_extent(d.H, d.ph, d.dh, d.R, d.sh);
    const int Q = out_extent(d.W, d.pw, d.dw, d.S, d.sw);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < d.N; ++n) {
        double *dxn = dx + (size_t)n * d.C * d.H * d.W;
        if (!accumulate) memset(dxn, 0, sizeof(double) * (size_t)d.C * d.H * d.W);
        for (int k = 0; k < d.K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    const double g = dy[(((size_t)n * d.K + k) * P + p) * Q + q];
                    for (int c = 0; c < d.C; ++c)
                        for (int r = 0; r < d.R; ++r) {
                            const int h = p * d.sh - d.ph + r * d.dh;
                            if (h < 0 || h >= d.H) continue;
                            for (int s = 0; s < d.S; ++s) {
                                const int v = q * d.sw - d.pw + s * d.dw;
                                if (v < 0 || v >= d.W) continue;
                                dxn[((size_t)c * d.H + h) * d.W + v] +=
                                    g * w[(((size_t)k * d.C + c) * d.R + r) * d.S + s];
                            }
                        }
                }
    }
}

/* dw[k,c,r,s] = sum_{n,p,q} dy[n,k,p,q] * x[n,c,p*sh-ph+r*dh,q*sw-pw+s*dw]. */
void oracle_conv2d_wgrad(const double *x, const double *dy, double *dw, const int32_t *dims,
                         int accumulate)
{
    const conv_dims d = *(const conv_dims *)dims;
    const int P = out_extent(d.H, d.ph, d.dh, d.R, d.sh);
    const int Q = out_extent(d.W, d.pw, d.dw, d.S, d.sw);
#pragma omp parallel for schedule(static)
    for (int k = 0; k < d.K; ++k)
        for (int c = 0; c < d.C; ++c)
            for (int r = 0; r < d.R; ++r)
                for (int s = 0; s < d.S; ++s) {
                    double acc = 0.0;
                    for (int n = 0; n < d.N; ++n)
                        for (int p = 0; p < P; ++p) {
                            const int h = p * d.sh - d.ph + r * d.dh;
                            if (h < 0 || h >= d.H) continue;
                            for (int q = 0; q < Q; ++q) {
                                const int v = q * d.sw - d.pw + s * d.dw;
                                if (v < 0 || v >= d.W) continue;
                                acc += dy[(((size_t)n * d.K + k) * P + p) * Q + q] *
                                       x[(((size_t)n * d.C + c) * d.H + h) * d.W + v];
                            }
                        }
                    double *o = &dw[(((size_t)k * d.C + c) * d.R + r) * d.S + s];
                    *o = accumulate ? *o + acc : acc;
                }
}

/* The same three definitions evaluated only at listed output coordinates, for
 * shapes whose full evaluation would take minutes.  Each output element is an
 * independent sum, so this is the definition, not an approximation. */
void oracle_conv2d_fwd_at(const double *x, const double *w, const int32_t *dims, int64_t count,
                          const int32_t *nkpq, double *out)
{
    const conv_dims d = *(const conv_dims *)dims;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        const int n = nkpq[4 * i], k = nkpq[4 * i + 1], p = nkpq[4 * i + 2], q = nkpq[4 * i + 3];
        double acc = 0.0;
        for (int c = 0; c < d.C; ++c)
            for (int r = 0; r < d.R; ++r) {
                const int h = p * d.sh - d.ph + r * d.dh;
                if (h < 0 || h >= d.H) continue;
                for (int s = 0; s < d.S; ++s) {
                    const int v = q * d.sw - d.pw + s * d.dw;
                    if (v < 0 || v >= d.W) continue;
                    acc += x[(((size_t)n * d.C + c) * d.H + h) * d.W + v] *
                           w[(((size_t)k * d.C + c) * d.R + r) * d.S + s];
                }
            }
        out[i] = acc;
    }
}

/* dx[n,c,h,v] collects dy[n,k,p,q]*w[k,c,r,s] from every (p,r) with
 * p*sh-ph+r*dh == h and every (q,s) with q*sw-pw+s*dw == v. */
void oracle_conv2d_dgrad_at(const double *dy, const double *w, const int32_t *dims, int64_t count,
                            const int32_t *nchw, double *out)
{
    const conv_dims d = *(const conv_dims *)dims;
    const int P = out_extent(d.H, d.ph, d.dh, d.R, d.sh);
    const int Q = out_extent(d.W, d.pw, d.dw, d.S, d.sw);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        const int n = nchw[4 * i], c = nchw[4 * i + 1], h = nchw[4 * i + 2], v = nchw[4 * i + 3];
        double acc = 0.0;
        for (int r = 0; r < d.R; ++r) {
            const int th = h + d.ph - r * d.dh;
            if (th < 0 || th % d.sh != 0 || th / d.sh >= P) continue;
            const int p = th / d.sh;
            for (int s = 0; s < d.S; ++s) {
                const int tv = v + d.pw - s * d.dw;
                if (tv < 0 || tv % d.sw != 0 || tv / d.sw >= Q) continue;
                const int q = tv / d.sw;
                for (int k = 0; k < d.K; ++k)
                    acc += dy[(((size_t)n * d.K + k) * P + p) * Q + q] *
                           w[(((size_t)k * d.C + c) * d.R + r) * d.S + s];
            }
        }
        out[i] = acc;
    }
}

void oracle_conv2d_wgrad_at(const double *x, const double *dy, const int32_t *dims, int64_t count,
                            const int32_t *kcrs, double *out)
{
    const conv_dims d = *(const conv_dims *)dims;
    const int P = out_extent(d.H, d.ph, d.dh, d.R, d.sh);
    const int Q = out_extent(d.W, d.pw, d.dw, d.S, d.sw);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < count; ++i) {
        const int k = kcrs[4 * i], c = kcrs[4 * i + 1], r = kcrs[4 * i + 2], s = kcrs[4 * i + 3];
        double acc = 0.0;
        for (int n = 0; n < d.N; ++n)
            for (int p = 0; p < P; ++p) {
                const int h = p * d.sh - d.ph + r * d.dh;
                if (h < 0 || h >= d.H) continue;
                for (int q = 0; q < Q; ++q) {
                    const int v = q * d.sw - d.pw + s * d.dw;
                    if (v < 0 || v >= d.W) continue;
                    acc += dy[(((size_t)n * d.K + k) * P + p) * Q + q] *
                           x[(((size_t)n * d.C + c) * d.H + h) * d.W + v];
                }
            }
        out[i] = acc;
    }
}

/* Train-mode batch-norm over (n,h,w) per channel, then optional residual add,
 * then optional ReLU:
 *   mean = sum(x)/M, var = sum((x-mean)^2)/M (biased), invstd = 1/sqrt(var+eps)
 *   z = gamma*(x-mean)*invstd + beta (+ residual);  out = relu ? max(z,0) : z
 * Running statistics, when given, move by `momentum` toward the batch mean and
 * the unbiased batch variance (the usual framework convention). */
void oracle_bn_relu_add_fwd(const double *x, const double *residual, const double *gamma,
                            const double *beta, double *out, double *save_mean,
                            double *save_invstd, double *running_mean, double *running_var,
                            int N, int C, int H, int W, double eps, double momentum, int relu)
{
    const size_t HW = (size_t)H * W;
    const double M = (double)N * (double)HW;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        double sum = 0.0;
        for (int n = 0; n < N; ++n) {
            const double *px = x + ((size_t)n * C + c) * HW;
            for (size_t i = 0; i < HW; ++i) sum += px[i];
        }
        const double mean = sum / M;
        double ss = 0.0;
        for (int n = 0; n < N; ++n) {
            const double *px = x + ((size_t)n * C + c) * HW;
            for (size_t i = 0; i < HW; ++i) ss += (px[i] - mean) * (px[i] - mean);
        }
        const double var = ss / M;
        const double invstd = 1.0 / sqrt(var + eps);
        save_mean[c] = mean;
        save_invstd[c] = invstd;
        if (running_mean) running_mean[c] = (1.0 - momentum) * running_mean[c] + momentum * mean;
        if (running_var) {
            const double unbiased = M > 1.0 ? ss / (M - 1.0) : var;
            running_var[c] = (1.0 - momentum) * running_var[c] + momentum * unbiased;
        }
        for (int n = 0; n < N; ++n) {
            const size_t base = ((size_t)n * C + c) * HW;
            for (size_t i = 0; i < HW; ++i) {
                double z = gamma[c] * (x[base + i] - mean) * invstd + beta[c];
                if (residual) z += residual[base + i];
                out[base + i] = (relu && !(z > 0.0)) ? 0.0 : z;
            }
        }
    }
}

/* Backward of the above.  With xhat = (x-mean)*invstd and M = N*H*W:
 *   dz = relu ? dout*[out>0] : dout        (mask taken from the stored out)
 *   dbeta = sum dz,  dgamma = sum dz*xhat
 *   dx = gamma*invstd*(dz - dbeta/M - xhat*dgamma/M),  dresidual = dz */
void oracle_bn_relu_add_bwd(const double *x, const double *out, const double *dout,
                            const double *gamma, const double *save_mean,
                            const double *save_invstd, double *dx, double *dresidual,
                            double *dgamma, double *dbeta, int N, int C, int H, int W, int relu)
{
    const size_t HW = (size_t)H * W;
    const double M = (double)N * (double)HW;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        const double mean = save_mean[c], invstd = save_invstd[c];
        double sb = 0.0, sg = 0.0;
        for (int n = 0; n < N; ++n) {
            const size_t base = ((size_t)n * C + c) * HW;
            for (size_t i = 0; i < HW; ++i) {
                const double dz = (relu && !(out[base + i] > 0.0)) ? 0.0 : dout[base + i];
                sb += dz;
                sg += dz * (x[base + i] - mean) * invstd;
            }
        }
        dbeta[c] = sb;
        dgamma[c] = sg;
        for (int n = 0; n < N; ++n) {
            const size_t base = ((size_t)n * C + c) * HW;
            for (size_t i = 0; i < HW; ++i) {
                const double dz = (relu && !(out[base + i] > 0.0)) ? 0.0 : dout[base + i];
                const double xhat = (x[base + i] - mean) * invstd;
                dx[base + i] = gamma[c] * invstd * (dz - sb / M - xhat * sg / M);
                if (dresidual) dresidual[base + i] = dz;
            }
        }
    }
}

/* Window maximum with padding treated as minus infinity.  idx holds the window
 * position r*S+s of the FIRST maximum in row-major (r,s) order, or -1 for a
 * window that covers no input element (then y = -inf). */
void oracle_maxpool2d_fwd(const double *x, double *y, int8_t *idx, int N, int C, int H, int W,
                          int R, int S, int sh, int sw, int ph, int pw)
{
    const int P = out_extent(H, ph, 1, R, sh);
    const int Q = out_extent(W, pw, 1, S, sw);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            const double *px = x + ((size_t)n * C + c) * H * W;
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double best = -INFINITY;
                    int where = -1;
                    for (int r = 0; r < R; ++r) {
                        const int h = p * sh - ph + r;
                        if (h < 0 || h >= H) continue;
                        for (int s = 0; s < S; ++s) {
                            const int v = q * sw - pw + s;
                            if (v < 0 || v >= W) continue;
                            const double val = px[(size_t)h * W + v];
                            if (where < 0 || val > best) {
                                best = val;
                                where = r * S + s;
                            }
                        }
                    }
                    const size_t o = (((size_t)n * C + c) * P + p) * Q + q;
                    y[o] = best;
                    idx[o] = (int8_t)where;
                }
        }
}

/* dx starts at zero; every output window sends its dy to the input element
 * idx names.  Windows overlap when stride < window, so contributions add. */
void oracle_maxpool2d_bwd(const double *dy, const int8_t *idx, double *dx, int N, int C, int H,
                          int W, int R, int S, int sh, int sw, int ph, int pw)
{
    const int P = out_extent(H, ph, 1, R, sh);
    const int Q = out_extent(W, pw, 1, S, sw);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            double *pd = dx + ((size_t)n * C + c) * H * W;
            memset(pd, 0, sizeof(double) * (size_t)H * W);
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    const size_t o = (((size_t)n * C + c) * P + p) * Q + q;
                    const int where = idx[o];
                    if (where < 0) continue;
                    const int h = p * sh - ph + where / S;
                    const int v = q * sw - pw + where % S;
                    pd[(size_t)h * W + v] += dy[o];
                }
        }
}

/* Round each value to the nearest bfloat16 (8 significant bits, the fp32
 * exponent range, ties to even), returned as a double.  Works from the exact
 * double, so there is no intermediate fp32 rounding. */
void oracle_round_bf16(const double *in, double *out, int64_t count)
{
    const double max_bf16 = 0x1.FEp127; /* (2 - 2^-7) * 2^127 */
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        const double v = in[i];
        if (v == 0.0 || !isfinite(v)) {
            out[i] = v;
            continue;
        }
        int e;
        (void)frexp(v, &e);          /* |v| = m * 2^e with m in [0.5, 1) */
        int quantum = e - 8;         /* keep 8 significant bits */
        if (quantum < -133) quantum = -133; /* bf16 subnormal spacing 2^-133 */
        double r = ldexp(nearbyint(ldexp(v, -quantum)), quantum); /* default mode: ties to even */
        if (fabs(r) > max_bf16) r = copysign(INFINITY, v);
        out[i] = r;
    }
}

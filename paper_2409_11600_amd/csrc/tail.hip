// The operations that close a training step behind the residual blocks: global average pool and fully connected
// layer (the head of the ResNet recipe the paper trains, section "Experiments and Discussion"; the fully connected
// layer is the `@` operator of section "Automatic Differentiation"), the softmax cross-entropy loss node that has to
// end every step (same section), and the optimizer updates with the clearing of the gradient buffers (section
// "Caching and Pooling").  All of them are small and bound by memory or by launch latency; the kernels are plain
// streaming code.  The fully connected layer runs on the convolution kernels (1x1 filter, 1x1 image).
#include <math.h>

#include "nsk_internal.h"

namespace nsk {
namespace {

bool unaligned(const void *p) { return ((uintptr_t)p & 15) != 0; }

#define TAIL_TRY(expr)                \
    do {                              \
        int status_ = (expr);         \
        if (status_ != NSK_OK) return status_; \
    } while (0)

__device__ inline float ld(const float *p, long i) { return p[i]; }
__device__ inline float ld(const bf16_t *p, long i) { return (float)p[i]; }

__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ inline float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// ----------------------------------------------------------------------------- global average pool
// NHWC, channel count a multiple of the 16-byte vector width with C/VEC dividing 1024: one block of 1024 threads per
// image.  A thread owns one vector of channels and every G-th position (G = 1024 / vectors per pixel), four loads
// in flight; the G partial sums per channel meet in LDS and are added in a fixed order.
template <typename T, int VEC>
__global__ __launch_bounds__(1024) void avgpool_fwd_nhwc_vec(const T *__restrict__ x, T *__restrict__ y, int C, int HW)
{
    typedef T Vec __attribute__((ext_vector_type(VEC)));
    extern __shared__ float part[];                 // [G][C]
    const int CV = C / VEC, G = 1024 / CV;
    const int cv = threadIdx.x % CV, g = threadIdx.x / CV;
    const Vec *p = (const Vec *)(x + (long)blockIdx.x * HW * C) + cv;
    float s[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) s[e] = 0.f;
    int k = g;
    for (; k + 3 * G < HW; k += 4 * G) {
        const Vec v0 = p[(long)k * CV], v1 = p[(long)(k + G) * CV], v2 = p[(long)(k + 2 * G) * CV], v3 = p[(long)(k + 3 * G) * CV];
#pragma unroll
        for (int e = 0; e < VEC; ++e) s[e] += ((float)v0[e] + (float)v1[e]) + ((float)v2[e] + (float)v3[e]);
    }
    for (; k < HW; k += G) {
        const Vec v = p[(long)k * CV];
#pragma unroll
        for (int e = 0; e < VEC; ++e) s[e] += (float)v[e];
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) part[g * C + cv * VEC + e] = s[e];
    __syncthreads();
    for (int c = threadIdx.x; c < C; c += 1024) {
        float t = 0.f;
        for (int gg = 0; gg < G; ++gg) t += part[gg * C + c];
        y[(long)blockIdx.x * C + c] = (T)(t / (float)HW);
    }
}
// NHWC, any channel count: one thread per (n, c), neighbouring threads read neighbouring channels.
template <typename T>
__global__ __launch_bounds__(256) void avgpool_fwd_nhwc(const T *__restrict__ x, T *__restrict__ y, int N, int C, int HW)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= (long)N * C) return;
    const long n = i / C, c = i - n * C;
    const T *p = x + n * HW * (long)C + c;
    float s = 0.f;
    for (int k = 0; k < HW; ++k) s += ld(p, (long)k * C);
    y[i] = (T)(s / (float)HW);
}
// NCHW: one wavefront per (n, c) plane, lanes stride over the plane, fixed-order cross-lane sum.
template <typename T>
__global__ __launch_bounds__(256) void avgpool_fwd_nchw(const T *__restrict__ x, T *__restrict__ y, long planes, int HW)
{
    const long pl = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (pl >= planes) return;
    const T *p = x + pl * HW;
    float s = 0.f;
    for (int k = threadIdx.x & 63; k < HW; k += 64) s += ld(p, k);
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) y[pl] = (T)(s / (float)HW);
}
template <typename T, bool NHWC>
__global__ __launch_bounds__(256) void avgpool_bwd_kernel(const T *__restrict__ dy, T *__restrict__ dx, long total, int C,
                                                          int HW, int accumulate)
{
    const float inv = 1.f / (float)HW;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        long nc;
        if (NHWC) {
            const long n = i / ((long)HW * C);
            nc = n * C + i % C;
        } else {
            nc = i / HW;
        }
        float v = ld(dy, nc) * inv;
        if (accumulate) v += ld(dx, i);
        dx[i] = (T)v;
    }
}

// ----------------------------------------------------------------------------- fully connected layer helpers
template <typename T>
__global__ __launch_bounds__(256) void add_bias_kernel(T *__restrict__ y, const float *__restrict__ bias, long total, int K)
{
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256)
        y[i] = (T)(ld(y, i) + bias[i % K]);
}
// db[k] (+)= sum_n dy[n][k]: a block owns 64 columns (lane = column, so a wavefront reads contiguous bytes of a row),
// its 16 wavefronts take every 16th row each and their partial sums are added in a fixed order.
template <typename T>
__global__ __launch_bounds__(1024) void bias_grad_kernel(const T *__restrict__ dy, float *__restrict__ db, int N, int K,
                                                         int accumulate)
{
    __shared__ float part[16][64];
    const int lane = threadIdx.x & 63, rl = threadIdx.x >> 6, k = blockIdx.x * 64 + lane;
    float s = 0.f;
    if (k < K) {
#pragma unroll 8
        for (int n = rl; n < N; n += 16) s += ld(dy, (long)n * K + k);
    }
    part[rl][lane] = s;
    __syncthreads();
    if (rl == 0 && k < K) {
        float t = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) t += part[r][lane];
        db[k] = accumulate ? db[k] + t : t;
    }
}

// Matrix products with very few rows (a recurrent step: 50 samples): a tile kernel would run on a handful of blocks,
// so here every output element has its own thread and the product runs on the vector units.
//   forward:  y[n][k] = sum_c x[n][c] * w[k][c] (+ bias[k]); lane = k (the 64 rows of w a wavefront walks stay in L1
//             for the iterations that share a cache line)
//   backward: dx[n][c] (+)= sum_k dy[n][k] * w[k][c]; lane = c, w read row by row with consecutive lanes on
//             consecutive c, so no packed transposed copy of the filter is needed
// forward: one thread per output element (splitting its reduction over wavefronts, as the backward kernel below does,
// is slower here: four times as many wavefronts then walk the rows of w with a stride)
template <typename T>
__global__ __launch_bounds__(256) void linear_small_fwd_kernel(const T *__restrict__ x, const T *__restrict__ w,
                                                               const float *__restrict__ bias, T *__restrict__ y, int N,
                                                               int C, int K)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= (long)N * K) return;
    const int n = (int)(i / K), k = (int)(i - (long)n * K);
    const T *xr = x + (long)n * C, *wr = w + (long)k * C;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    int c = 0;
    for (; c + 3 < C; c += 4) {
        s0 += ld(xr, c) * ld(wr, c);
        s1 += ld(xr, c + 1) * ld(wr, c + 1);
        s2 += ld(xr, c + 2) * ld(wr, c + 2);
        s3 += ld(xr, c + 3) * ld(wr, c + 3);
    }
    for (; c < C; ++c) s0 += ld(xr, c) * ld(wr, c);
    float r = (s0 + s1) + (s2 + s3);
    if (bias) r = (float)(T)r + bias[k];      // as the large path: product rounded to the storage type, then the bias
    y[i] = (T)r;
}

// backward: a block computes 64 consecutive outputs of one row; its four wavefronts each take a quarter of the
// reduction and the quarters are added in a fixed order through LDS.  (Giving a block several rows, so that a weight
// element is loaded once for all of them, was measured slower: 16 us against 9 us at 50 rows x 768 -> 256, because the
// launch then has too few blocks to hide the latency of its loads.)
template <typename T>
__global__ __launch_bounds__(256) void linear_small_dgrad_kernel(const T *__restrict__ dy, const T *__restrict__ w,
                                                                 T *__restrict__ dx, int N, int C, int K, int accumulate)
{
    __shared__ float part[4][64];
    const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int n = blockIdx.y, c = blockIdx.x * 64 + lane;
    const int k0 = (int)((long)K * q / 4), k1 = (int)((long)K * (q + 1) / 4);
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    if (c < C) {
        const T *dr = dy + (long)n * K, *wc = w + c;
        int k = k0;
        for (; k + 3 < k1; k += 4) {
            s0 += ld(dr, k) * ld(wc, (long)k * C);
            s1 += ld(dr, k + 1) * ld(wc, (long)(k + 1) * C);
            s2 += ld(dr, k + 2) * ld(wc, (long)(k + 2) * C);
            s3 += ld(dr, k + 3) * ld(wc, (long)(k + 3) * C);
        }
        for (; k < k1; ++k) s0 += ld(dr, k) * ld(wc, (long)k * C);
    }
    part[q][lane] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    if (q == 0 && c < C) {
        float r = (part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane]);
        const long i = (long)n * C + c;
        if (accumulate) r += ld(dx, i);
        dx[i] = (T)r;
    }
}

constexpr int kSmallRows = 64;     // up to this many rows the per-element kernels are used

// ----------------------------------------------------------------------------- softmax cross-entropy
// One wavefront per sample.  mode 0: per-sample loss; mode 1: gradient of the logits.
template <typename T, int MODE>
__global__ __launch_bounds__(256) void xent_kernel(const T *__restrict__ z, const int *__restrict__ labels, int N, int K,
                                                   float *__restrict__ per_sample, T *__restrict__ dz, float coef)
{
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;
    const int lane = threadIdx.x & 63;
    const T *row = z + (long)n * K;
    float m = -INFINITY;
    for (int k = lane; k < K; k += 64) m = fmaxf(m, ld(row, k));
    m = wave_max(m);
    float s = 0.f;
    for (int k = lane; k < K; k += 64) s += expf(ld(row, k) - m);
    s = wave_sum(s);
    const int lab = labels[n];
    if (MODE == 0) {
        if (lane == 0) per_sample[n] = (lab >= 0 && lab < K) ? logf(s) + (m - ld(row, lab)) : NAN;
    } else {
        const float inv = 1.f / s;
        for (int k = lane; k < K; k += 64) {
            const float p = expf(ld(row, k) - m) * inv;
            dz[(long)n * K + k] = (T)(coef * (p - (k == lab ? 1.f : 0.f)));
        }
    }
}
// loss = mean of per_sample, one block, fixed order.
__global__ __launch_bounds__(256) void mean_kernel(const float *__restrict__ v, int N, float *__restrict__ out)
{
    __shared__ double part[4];
    double s = 0.0;
    for (int i = threadIdx.x; i < N; i += 256) s += (double)v[i];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) out[0] = (float)(((part[0] + part[1]) + (part[2] + part[3])) / (double)N);
}

// ----------------------------------------------------------------------------- optimizers
struct AdamCoef {
    float lr, beta1, beta2, eps, c1, c2;   // c1 = 1/(1-beta1^t); c2 = 1/(1-beta2^t)
};

// One launch updates up to kMaxParams parameter tensors: blockIdx.y names the tensor, blockIdx.x strides over it.
constexpr int kMaxParams = 32;
struct ParamEntry {
    float *w, *g, *s1, *s2;
    bf16_t *w_lp;
    size_t n;
    float wd;        // SGD: weight decay; AdamW: 1 - lr*weight_decay
};
struct ParamTable {
    ParamEntry e[kMaxParams];
};

template <bool ADAM>
__global__ __launch_bounds__(256) void optimizer_kernel(const ParamTable tab, float lr, float momentum, AdamCoef ac,
                                                        const float *__restrict__ grad_scale)
{
    const ParamEntry &p = tab.e[blockIdx.y];
    const size_t n = p.n;
    float *__restrict__ w = p.w, *__restrict__ g = p.g, *__restrict__ s1 = p.s1, *__restrict__ s2 = p.s2;
    bf16_t *__restrict__ w_lp = p.w_lp;
    const float wd = p.wd;
    const float scale = grad_scale ? grad_scale[0] : 1.f;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        float wi = w[i];
        const float gi = g[i] * scale;
        if (ADAM) {
            wi *= wd;
            const float m = ac.beta1 * s1[i] + (1.f - ac.beta1) * gi;
            const float v = ac.beta2 * s2[i] + (1.f - ac.beta2) * gi * gi;
            s1[i] = m;
            s2[i] = v;
            wi -= ac.lr * (m * ac.c1) / (sqrtf(v * ac.c2) + ac.eps);
        } else {
            const float v = momentum * s1[i] + (gi + wd * wi);
            s1[i] = v;
            wi -= lr * v;
        }
        w[i] = wi;
        g[i] = 0.f;
        if (w_lp) w_lp[i] = (bf16_t)wi;
    }
}

__global__ __launch_bounds__(256) void sumsq_partial_kernel(size_t n, const float *__restrict__ g, float *__restrict__ partials)
{
    __shared__ double part[4];
    double s = 0.0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const float v = g[i];
        s += (double)(v * v);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) partials[blockIdx.x] = (float)((part[0] + part[1]) + (part[2] + part[3]));
}
__global__ void sumsq_final_kernel(const float *__restrict__ partials, int nb, float *__restrict__ sumsq)
{
    double s = 0.0;
    for (int i = 0; i < nb; ++i) s += (double)partials[i];
    sumsq[0] = (float)((double)sumsq[0] + s);
}
__global__ void clip_scale_kernel(const float *__restrict__ sumsq, float max_norm, float *__restrict__ scale)
{
    const float r = max_norm / (sqrtf(sumsq[0]) + 1e-6f);
    scale[0] = r < 1.f ? r : 1.f;
}

int stream_grid(size_t items)
{
    size_t b = (items + 255) / 256;
    if (b > 256 * 16) b = 256 * 16;
    if (b < 1) b = 1;
    return (int)b;
}

bool dtype_ok(int dtype) { return dtype == NSK_F32 || dtype == NSK_BF16; }

nsk_conv_desc_t linear_as_conv(const nsk_linear_desc_t *d)
{
    nsk_conv_desc_t c{};
    c.N = d->N; c.C = d->C; c.H = 1; c.W = 1;
    c.K = d->K; c.R = 1; c.S = 1;
    c.stride_h = c.stride_w = 1;
    c.pad_h = c.pad_w = 0;
    c.dil_h = c.dil_w = 1;
    c.dtype = d->dtype;
    c.layout = NSK_NHWC;
    return c;
}

int linear_check(const nsk_linear_desc_t *d)
{
    if (!d) return NSK_ERR_NULL;
    if (d->N <= 0 || d->C <= 0 || d->K <= 0 || !dtype_ok(d->dtype)) return NSK_ERR_BAD_DESC;
    return NSK_OK;
}

}  // namespace
}  // namespace nsk

using namespace nsk;

extern "C" {

int nsk_global_avgpool_fwd(int dtype, int layout, int N, int C, int H, int W, const void *x, void *y, void *stream)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || !dtype_ok(dtype) || (layout != NSK_NCHW && layout != NSK_NHWC))
        return NSK_ERR_BAD_DESC;
    if (!x || !y) return NSK_ERR_NULL;
    if (unaligned(x) || unaligned(y)) return NSK_ERR_ALIGNMENT;
    hipStream_t st = (hipStream_t)stream;
    const long planes = (long)N * C;
    const int HW = H * W;
    const int vec = dtype == NSK_BF16 ? 8 : 4;
    if (layout == NSK_NHWC && C % vec == 0 && 1024 % (C / vec) == 0) {
        const size_t smem = (size_t)1024 * vec * sizeof(float);     // G * C floats with G = 1024 / (C / vec)
        if (dtype == NSK_BF16)
            hipLaunchKernelGGL((avgpool_fwd_nhwc_vec<bf16_t, 8>), dim3(N), dim3(1024), smem, st, (const bf16_t *)x, (bf16_t *)y, C, HW);
        else
            hipLaunchKernelGGL((avgpool_fwd_nhwc_vec<float, 4>), dim3(N), dim3(1024), smem, st, (const float *)x, (float *)y, C, HW);
    } else if (layout == NSK_NHWC) {
        const dim3 grid((unsigned)((planes + 255) / 256));
        if (dtype == NSK_BF16)
            hipLaunchKernelGGL(avgpool_fwd_nhwc<bf16_t>, grid, dim3(256), 0, st, (const bf16_t *)x, (bf16_t *)y, N, C, HW);
        else
            hipLaunchKernelGGL(avgpool_fwd_nhwc<float>, grid, dim3(256), 0, st, (const float *)x, (float *)y, N, C, HW);
    } else {
        const dim3 grid((unsigned)((planes + 3) / 4));
        if (dtype == NSK_BF16)
            hipLaunchKernelGGL(avgpool_fwd_nchw<bf16_t>, grid, dim3(256), 0, st, (const bf16_t *)x, (bf16_t *)y, planes, HW);
        else
            hipLaunchKernelGGL(avgpool_fwd_nchw<float>, grid, dim3(256), 0, st, (const float *)x, (float *)y, planes, HW);
    }
    return check_launch();
}

int nsk_global_avgpool_bwd(int dtype, int layout, int N, int C, int H, int W, const void *dy, void *dx, int accumulate,
                           void *stream)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || !dtype_ok(dtype) || (layout != NSK_NCHW && layout != NSK_NHWC))
        return NSK_ERR_BAD_DESC;
    if (accumulate != 0 && accumulate != 1) return NSK_ERR_BAD_DESC;
    if (!dy || !dx) return NSK_ERR_NULL;
    if (unaligned(dy) || unaligned(dx)) return NSK_ERR_ALIGNMENT;
    hipStream_t st = (hipStream_t)stream;
    const long total = (long)N * C * H * W;
    const dim3 grid(stream_grid((size_t)total));
#define NSK_AP(T, L) \
    hipLaunchKernelGGL((avgpool_bwd_kernel<T, L>), grid, dim3(256), 0, st, (const T *)dy, (T *)dx, total, C, H * W, accumulate)
    if (dtype == NSK_BF16) {
        if (layout == NSK_NHWC) NSK_AP(bf16_t, true); else NSK_AP(bf16_t, false);
    } else {
        if (layout == NSK_NHWC) NSK_AP(float, true); else NSK_AP(float, false);
    }
#undef NSK_AP
    return check_launch();
}

size_t nsk_linear_workspace_bytes(const nsk_linear_desc_t *desc, int pass)
{
    if (linear_check(desc) != NSK_OK) return 0;
    const nsk_conv_desc_t c = linear_as_conv(desc);
    return nsk_conv2d_workspace_bytes(&c, pass);
}

int nsk_linear_fwd(const nsk_linear_desc_t *desc, const void *x, const void *w, const float *bias, void *y,
                   void *workspace, size_t workspace_bytes, void *stream)
{
    TAIL_TRY(linear_check(desc));
    if (bias && unaligned(bias)) return NSK_ERR_ALIGNMENT;
    if (desc->N <= kSmallRows) {
        if (!x || !w || !y) return NSK_ERR_NULL;
        if (unaligned(x) || unaligned(w) || unaligned(y)) return NSK_ERR_ALIGNMENT;
        const long total = (long)desc->N * desc->K;
        const dim3 grid((unsigned)((total + 255) / 256));
        if (desc->dtype == NSK_BF16)
            hipLaunchKernelGGL(linear_small_fwd_kernel<bf16_t>, grid, dim3(256), 0, (hipStream_t)stream, (const bf16_t *)x,
                               (const bf16_t *)w, bias, (bf16_t *)y, desc->N, desc->C, desc->K);
        else
            hipLaunchKernelGGL(linear_small_fwd_kernel<float>, grid, dim3(256), 0, (hipStream_t)stream, (const float *)x,
                               (const float *)w, bias, (float *)y, desc->N, desc->C, desc->K);
        return check_launch();
    }
    const nsk_conv_desc_t c = linear_as_conv(desc);
    TAIL_TRY(nsk_conv2d_fwd(&c, x, w, y, workspace, workspace_bytes, stream));
    if (bias) {
        const long total = (long)desc->N * desc->K;
        const dim3 grid(stream_grid((size_t)total));
        if (desc->dtype == NSK_BF16)
            hipLaunchKernelGGL(add_bias_kernel<bf16_t>, grid, dim3(256), 0, (hipStream_t)stream, (bf16_t *)y, bias, total, desc->K);
        else
            hipLaunchKernelGGL(add_bias_kernel<float>, grid, dim3(256), 0, (hipStream_t)stream, (float *)y, bias, total, desc->K);
        return check_launch();
    }
    return NSK_OK;
}

int nsk_linear_dgrad(const nsk_linear_desc_t *desc, const void *dy, const void *w, void *dx, int accumulate,
                     void *workspace, size_t workspace_bytes, void *stream)
{
    TAIL_TRY(linear_check(desc));
    if (desc->N <= kSmallRows) {
        if (accumulate != 0 && accumulate != 1) return NSK_ERR_BAD_DESC;
        if (!dy || !w || !dx) return NSK_ERR_NULL;
        if (unaligned(dy) || unaligned(w) || unaligned(dx)) return NSK_ERR_ALIGNMENT;
        const dim3 grid((unsigned)((desc->C + 63) / 64), (unsigned)desc->N);
        if (desc->dtype == NSK_BF16)
            hipLaunchKernelGGL(linear_small_dgrad_kernel<bf16_t>, grid, dim3(256), 0, (hipStream_t)stream, (const bf16_t *)dy,
                               (const bf16_t *)w, (bf16_t *)dx, desc->N, desc->C, desc->K, accumulate);
        else
            hipLaunchKernelGGL(linear_small_dgrad_kernel<float>, grid, dim3(256), 0, (hipStream_t)stream, (const float *)dy,
                               (const float *)w, (float *)dx, desc->N, desc->C, desc->K, accumulate);
        return check_launch();
    }
    const nsk_conv_desc_t c = linear_as_conv(desc);
    return nsk_conv2d_dgrad(&c, dy, w, dx, accumulate, workspace, workspace_bytes, stream);
}

int nsk_linear_wgrad(const nsk_linear_desc_t *desc, const void *x, const void *dy, float *dw, float *db, int accumulate,
                     void *workspace, size_t workspace_bytes, void *stream)
{
    TAIL_TRY(linear_check(desc));
    if (db && unaligned(db)) return NSK_ERR_ALIGNMENT;
    const nsk_conv_desc_t c = linear_as_conv(desc);
    TAIL_TRY(nsk_conv2d_wgrad(&c, x, dy, dw, accumulate, workspace, workspace_bytes, stream));
    if (db) {
        const dim3 grid((unsigned)((desc->K + 63) / 64));
        if (desc->dtype == NSK_BF16)
            hipLaunchKernelGGL(bias_grad_kernel<bf16_t>, grid, dim3(1024), 0, (hipStream_t)stream, (const bf16_t *)dy, db, desc->N,
                               desc->K, accumulate);
        else
            hipLaunchKernelGGL(bias_grad_kernel<float>, grid, dim3(1024), 0, (hipStream_t)stream, (const float *)dy, db, desc->N,
                               desc->K, accumulate);
        return check_launch();
    }
    return NSK_OK;
}

int nsk_transpose2d(int dtype, int rows, int cols, const void *src, void *dst, void *stream)
{
    if (rows <= 0 || cols <= 0 || !dtype_ok(dtype)) return NSK_ERR_BAD_DESC;
    if (!src || !dst) return NSK_ERR_NULL;
    if (unaligned(src) || unaligned(dst)) return NSK_ERR_ALIGNMENT;
    // [rows][cols] -> [cols][rows] is the NHWC -> NCHW copy of one image with rows pixels and cols channels
    return launch_nhwc_to_nchw(dtype, src, dst, 1, cols, rows, 1, 0, (hipStream_t)stream);
}

int nsk_softmax_xent_fwd(int dtype, int N, int K, const void *logits, const int *labels, float *per_sample, float *loss,
                         void *stream)
{
    if (N <= 0 || K <= 0 || !dtype_ok(dtype)) return NSK_ERR_BAD_DESC;
    if (!logits || !labels || !per_sample || !loss) return NSK_ERR_NULL;
    if (unaligned(logits) || unaligned(labels) || unaligned(per_sample) || unaligned(loss)) return NSK_ERR_ALIGNMENT;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid((unsigned)((N + 3) / 4));
    if (dtype == NSK_BF16)
        hipLaunchKernelGGL((xent_kernel<bf16_t, 0>), grid, dim3(256), 0, st, (const bf16_t *)logits, labels, N, K, per_sample,
                           (bf16_t *)nullptr, 0.f);
    else
        hipLaunchKernelGGL((xent_kernel<float, 0>), grid, dim3(256), 0, st, (const float *)logits, labels, N, K, per_sample,
                           (float *)nullptr, 0.f);
    hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(256), 0, st, per_sample, N, loss);
    return check_launch();
}

int nsk_softmax_xent_bwd(int dtype, int N, int K, const void *logits, const int *labels, float dloss, void *dlogits,
                         void *stream)
{
    if (N <= 0 || K <= 0 || !dtype_ok(dtype)) return NSK_ERR_BAD_DESC;
    if (!logits || !labels || !dlogits) return NSK_ERR_NULL;
    if (unaligned(logits) || unaligned(labels) || unaligned(dlogits)) return NSK_ERR_ALIGNMENT;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid((unsigned)((N + 3) / 4));
    const float coef = dloss / (float)N;
    if (dtype == NSK_BF16)
        hipLaunchKernelGGL((xent_kernel<bf16_t, 1>), grid, dim3(256), 0, st, (const bf16_t *)logits, labels, N, K,
                           (float *)nullptr, (bf16_t *)dlogits, coef);
    else
        hipLaunchKernelGGL((xent_kernel<float, 1>), grid, dim3(256), 0, st, (const float *)logits, labels, N, K,
                           (float *)nullptr, (float *)dlogits, coef);
    return check_launch();
}

// Validates one parameter record and appends it to the launch table.
static int add_param(const nsk_param_t &q, bool adam, float wd_field, ParamTable *tab, int slot, size_t *max_n)
{
    if (q.n == 0) return NSK_ERR_BAD_DESC;
    if (!q.w || !q.grad || !q.state1 || (adam && !q.state2)) return NSK_ERR_NULL;
    if (unaligned(q.w) || unaligned(q.grad) || unaligned(q.state1) || (adam && unaligned(q.state2)) || (q.w_lp && unaligned(q.w_lp)))
        return NSK_ERR_ALIGNMENT;
    ParamEntry &e = tab->e[slot];
    e.w = q.w; e.g = q.grad; e.s1 = q.state1; e.s2 = adam ? q.state2 : nullptr;
    e.w_lp = (bf16_t *)q.w_lp;
    e.n = q.n;
    e.wd = wd_field;
    if (q.n > *max_n) *max_n = q.n;
    return NSK_OK;
}

static int optimizer_launch(bool adam, int count, const nsk_param_t *params, float lr, float momentum, AdamCoef ac,
                            const float *grad_scale, void *stream)
{
    if (count <= 0) return NSK_ERR_BAD_DESC;
    if (!params) return NSK_ERR_NULL;
    if (grad_scale && ((uintptr_t)grad_scale & 3)) return NSK_ERR_ALIGNMENT;
    // validate everything before the first launch
    for (int i = 0; i < count; ++i) {
        ParamTable scratch;
        size_t mx = 0;
        TAIL_TRY(add_param(params[i], adam, 0.f, &scratch, 0, &mx));
    }
    for (int base = 0; base < count; base += kMaxParams) {
        const int m = count - base < kMaxParams ? count - base : kMaxParams;
        ParamTable tab{};
        size_t max_n = 0;
        for (int i = 0; i < m; ++i) {
            const nsk_param_t &q = params[base + i];
            TAIL_TRY(add_param(q, adam, adam ? 1.f - lr * q.weight_decay : q.weight_decay, &tab, i, &max_n));
        }
        size_t bx = (max_n + 255) / 256;
        if (bx > 1024) bx = 1024;
        const dim3 grid((unsigned)bx, (unsigned)m);
        if (adam)
            hipLaunchKernelGGL(optimizer_kernel<true>, grid, dim3(256), 0, (hipStream_t)stream, tab, lr, 0.f, ac, grad_scale);
        else
            hipLaunchKernelGGL(optimizer_kernel<false>, grid, dim3(256), 0, (hipStream_t)stream, tab, lr, momentum, ac, grad_scale);
    }
    return check_launch();
}

int nsk_sgd_momentum_step_multi(int count, const nsk_param_t *params, float lr, float momentum, const float *grad_scale,
                                void *stream)
{
    return optimizer_launch(false, count, params, lr, momentum, AdamCoef{}, grad_scale, stream);
}

int nsk_adamw_step_multi(int count, const nsk_param_t *params, int step, float lr, float beta1, float beta2, float eps,
                         const float *grad_scale, void *stream)
{
    if (step < 1 || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f)) return NSK_ERR_BAD_DESC;
    AdamCoef ac;
    ac.lr = lr; ac.beta1 = beta1; ac.beta2 = beta2; ac.eps = eps;
    ac.c1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)step)));
    ac.c2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)step)));
    return optimizer_launch(true, count, params, lr, 0.f, ac, grad_scale, stream);
}

int nsk_sgd_momentum_step(size_t n, float *w, float *grad, float *velocity, void *w_lp, float lr, float momentum,
                          float weight_decay, const float *grad_scale, void *stream)
{
    const nsk_param_t p = {w, grad, velocity, nullptr, w_lp, n, weight_decay};
    return nsk_sgd_momentum_step_multi(1, &p, lr, momentum, grad_scale, stream);
}

int nsk_adamw_step(size_t n, float *w, float *grad, float *m, float *v, void *w_lp, int step, float lr, float beta1,
                   float beta2, float eps, float weight_decay, const float *grad_scale, void *stream)
{
    const nsk_param_t p = {w, grad, m, v, w_lp, n, weight_decay};
    return nsk_adamw_step_multi(1, &p, step, lr, beta1, beta2, eps, grad_scale, stream);
}

int nsk_sumsq_accumulate(size_t n, const float *g, float *partials, float *sumsq, void *stream)
{
    if (n == 0) return NSK_ERR_BAD_DESC;
    if (!g || !partials || !sumsq) return NSK_ERR_NULL;
    if (unaligned(g) || unaligned(partials) || ((uintptr_t)sumsq & 3)) return NSK_ERR_ALIGNMENT;
    size_t nb = (n + 1023) / 1024;
    if (nb > NSK_SUMSQ_PARTIALS) nb = NSK_SUMSQ_PARTIALS;
    hipLaunchKernelGGL(sumsq_partial_kernel, dim3((unsigned)nb), dim3(256), 0, (hipStream_t)stream, n, g, partials);
    hipLaunchKernelGGL(sumsq_final_kernel, dim3(1), dim3(1), 0, (hipStream_t)stream, partials, (int)nb, sumsq);
    return check_launch();
}

int nsk_clip_scale(const float *sumsq, float max_norm, float *scale, void *stream)
{
    if (!sumsq || !scale) return NSK_ERR_NULL;
    if (!(max_norm > 0.f)) return NSK_ERR_BAD_DESC;
    if (((uintptr_t)sumsq & 3) || ((uintptr_t)scale & 3)) return NSK_ERR_ALIGNMENT;
    hipLaunchKernelGGL(clip_scale_kernel, dim3(1), dim3(1), 0, (hipStream_t)stream, sumsq, max_norm, scale);
    return check_launch();
}

}  // extern "C"

// Batch-norm (batch statistics) + residual add + ReLU, forward and backward, as HBM-streaming
// kernels.  The paper runs these element-wise steps unfused and names ReLU fusion as future work
// (conclusion); here each direction is one statistics pass and one fused apply pass:
//
//   forward : stats   x -> per-block partial sums          (read x)
//             finalize -> mean, invstd, scale, bias         (tiny)
//             apply   out = relu?(x*scale + bias [+ res])   (read x [,res], write out)
//   backward: reduce  dbeta, dgamma partials                (read x, out, dout)
//             finalize -> dbeta, dgamma, coefficients       (tiny)
//             apply   dx, dres                              (read x, out, dout; write dx [,dres])
//
// Statistics are accumulated in fp32 around a per-channel shift (the channel's first element), so
// E[(x-s)^2] - E[x-s]^2 does not cancel badly, and the per-block partials are combined in fp64 in
// a fixed order (reproducible, no atomics).
//
// Two code paths: a vectorised NHWC path (16-byte accesses, a thread keeps the same channels for
// all its rows) and a generic strided path that serves NCHW and channel counts the fast path
// cannot tile.
#include "nsk_internal.h"

namespace nsk {
namespace {

template <typename T> struct BT;
template <> struct BT<float> {
    static constexpr int VEC = 4;
    typedef f32x4 Vec;
};
template <> struct BT<bf16_t> {
    static constexpr int VEC = 8;
    typedef bf16x8 Vec;
};

__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Butterfly sum: every lane ends with the same value, combined in a fixed order.
__device__ inline double wave_sum_f64(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

bool nhwc_fast(const nsk_bn_desc_t &d)
{
    if (d.layout != NSK_NHWC) return false;
    const int VEC = d.dtype == NSK_BF16 ? 8 : 4;
    if (d.C % VEC) return false;
    const int cv = d.C / VEC;
    return cv <= 256 && 256 % cv == 0;
}

// ----------------------------------------------------------------------------- NHWC fast path

// Accumulates, per channel, sum(f0) and sum(f1) over the rows of this block, where (f0,f1) is
//   MODE 0 (forward stats):  (x - shift, (x - shift)^2)
//   MODE 1 (backward)     :  (dz, dz * xhat)
template <typename T, int MODE>
__global__ __launch_bounds__(256) void bn_reduce_nhwc(const T *__restrict__ x, const T *__restrict__ out,
                                                      const T *__restrict__ dout, const float *__restrict__ mean,
                                                      const float *__restrict__ invstd, int relu, long M, int C,
                                                      long rows_per_block, float *__restrict__ p0,
                                                      float *__restrict__ p1, unsigned char *__restrict__ mask,
                                                      const unsigned char *__restrict__ mask_in, int noshift = 0,
                                                      const float *__restrict__ act = nullptr)
{
    typedef typename BT<T>::Vec Vec;
    constexpr int VEC = BT<T>::VEC;
    const int CV = C / VEC, RP = 256 / CV;
    const int cv = threadIdx.x % CV, rr = threadIdx.x / CV;
    float s0[VEC], s1[VEC], sh[VEC], sc[VEC], as[VEC], ab[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        s0[e] = 0.f;
        s1[e] = 0.f;
        // act: the normalised activation was never stored (its consumers applied scale and shift on load): the ReLU
        // mask is recomputed from x with the same coefficients and the same expression
        as[e] = MODE == 1 && act ? act[cv * VEC + e] : 0.f;
        ab[e] = MODE == 1 && act ? act[C + cv * VEC + e] : 0.f;
        if (MODE == 0) {
            sh[e] = noshift ? 0.f : (float)x[cv * VEC + e];
            sc[e] = 1.f;
        } else {
            sh[e] = mean[cv * VEC + e];
            sc[e] = invstd[cv * VEC + e];
        }
    }
    const long r_begin = (long)blockIdx.x * rows_per_block;
    const long r_end = min(M, r_begin + rows_per_block);
#pragma unroll 4
    for (long r = r_begin + rr; r < r_end; r += RP) {
        const long off = r * C + cv * VEC;
        const Vec xv = *(const Vec *)(x + off);
        if (MODE == 0) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const float dlt = (float)xv[e] - sh[e];
                s0[e] += dlt;
                s1[e] += dlt * dlt;
            }
        } else {
            const Vec gv = *(const Vec *)(dout + off);
            unsigned bits = 0;
            if (mask_in) {
                bits = mask_in[off / VEC];        // handed over by the forward pass: `out` is not read at all
            } else if (act) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) bits |= ((float)(T)((float)xv[e] * as[e] + ab[e]) > 0.f ? 1u : 0u) << e;
                mask[off / VEC] = (unsigned char)bits;
            } else if (relu) {
                const Vec ov = *(const Vec *)(out + off);
#pragma unroll
                for (int e = 0; e < VEC; ++e) bits |= ((float)ov[e] > 0.f ? 1u : 0u) << e;
                // one byte per vector: the apply pass reads this instead of `out` (an eighth or a sixteenth of its bytes)
                mask[off / VEC] = (unsigned char)bits;
            }
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                float dz = (float)gv[e];
                if (relu && !((bits >> e) & 1u)) dz = 0.f;
                s0[e] += dz;
                s1[e] += dz * (((float)xv[e] - sh[e]) * sc[e]);
            }
        }
    }
    __shared__ float red0[256 * VEC], red1[256 * VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        red0[threadIdx.x * VEC + e] = s0[e];
        red1[threadIdx.x * VEC + e] = s1[e];
    }
    __syncthreads();
    // thread t < C sums column t over the RP row groups (row group rr holds channels at rr*C..)
    for (int c = threadIdx.x; c < C; c += 256) {
        float a0 = 0.f, a1 = 0.f;
        for (int g = 0; g < RP; ++g) {
            a0 += red0[g * C + c];
            a1 += red1[g * C + c];
        }
        p0[(long)blockIdx.x * C + c] = a0;
        p1[(long)blockIdx.x * C + c] = a1;
    }
}

template <typename T, bool HAS_RES, bool RELU>
__global__ __launch_bounds__(256) void bn_apply_nhwc(const T *__restrict__ x, const T *__restrict__ res,
                                                     T *__restrict__ out, const float *__restrict__ scale,
                                                     const float *__restrict__ bias, long nvec, int C,
                                                     unsigned char *__restrict__ mask)
{
    typedef typename BT<T>::Vec Vec;
    constexpr int VEC = BT<T>::VEC;
    // C/VEC divides 256 and the grid stride is a multiple of 256 vectors, so a thread always sees
    // the same VEC channels: their coefficients live in registers.
    const int c0 = (threadIdx.x % (C / VEC)) * VEC;
    float sc[VEC], bi[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        sc[e] = scale[c0 + e];
        bi[e] = bias[c0 + e];
    }
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (long)gridDim.x * 256) {
        const Vec xv = __builtin_nontemporal_load((const Vec *)(x + i * VEC));
        Vec rv;
        if (HAS_RES) rv = __builtin_nontemporal_load((const Vec *)(res + i * VEC));
        Vec ov;
        unsigned bits = 0;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            float z = (float)xv[e] * sc[e] + bi[e];
            if (HAS_RES) z += (float)rv[e];
            if (RELU) z = z > 0.f ? z : 0.f;
            ov[e] = (T)z;
            bits |= ((float)ov[e] > 0.f ? 1u : 0u) << e;   // of the value as stored
        }
        __builtin_nontemporal_store(ov, (Vec *)(out + i * VEC));
        if (RELU && mask) mask[i] = (unsigned char)bits;
    }
}

// dx = a*(dz - b - xhat*cc) with a = gamma*invstd, b = dbeta/M, cc = dgamma/M ; dres = dz
template <typename T, bool HAS_RES, bool RELU>
__global__ __launch_bounds__(256) void bn_bwd_apply_nhwc(const T *__restrict__ x, const T *__restrict__ out,
                                                         const T *__restrict__ dout, T *__restrict__ dx,
                                                         T *__restrict__ dres, const float *__restrict__ mean,
                                                         const float *__restrict__ invstd,
                                                         const float *__restrict__ coef, long nvec, int C,
                                                         const unsigned char *__restrict__ mask)
{
    typedef typename BT<T>::Vec Vec;
    constexpr int VEC = BT<T>::VEC;
    const int c0 = (threadIdx.x % (C / VEC)) * VEC;   // fixed per thread, see bn_apply_nhwc
    float mu[VEC], is[VEC], ka[VEC], kb[VEC], kc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        mu[e] = mean[c0 + e];
        is[e] = invstd[c0 + e];
        ka[e] = coef[c0 + e];
        kb[e] = coef[C + c0 + e];
        kc[e] = coef[2 * C + c0 + e];
    }
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (long)gridDim.x * 256) {
        const Vec xv = __builtin_nontemporal_load((const Vec *)(x + i * VEC));
        const Vec gv = __builtin_nontemporal_load((const Vec *)(dout + i * VEC));
        // ReLU mask of these VEC elements, written by the reduction pass (bit e set: out > 0)
        unsigned bits = ~0u;
        if (RELU) bits = __builtin_nontemporal_load(mask + i);
        Vec dxv, drv;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            float dz = (float)gv[e];
            if (RELU && !((bits >> e) & 1u)) dz = 0.f;
            const float xhat = ((float)xv[e] - mu[e]) * is[e];
            dxv[e] = (T)(ka[e] * (dz - kb[e] - xhat * kc[e]));
            drv[e] = (T)dz;
        }
        __builtin_nontemporal_store(dxv, (Vec *)(dx + i * VEC));
        if (HAS_RES) __builtin_nontemporal_store(drv, (Vec *)(dres + i * VEC));
    }
}

// ----------------------------------------------------------------------------- generic strided path
// element (n, c, s) lives at n*sn + c*sc + s*ss ; block (c, g) covers images [g*npg, (g+1)*npg)
template <typename T, int MODE>
__global__ __launch_bounds__(256) void bn_reduce_generic(const T *__restrict__ x, const T *__restrict__ out,
                                                         const T *__restrict__ dout, const float *__restrict__ mean,
                                                         const float *__restrict__ invstd, int relu, int N, long HW,
                                                         long sn, long scs, long ss, int npg, int C,
                                                         float *__restrict__ p0, float *__restrict__ p1, int noshift = 0)
{
    const int c = blockIdx.x, g = blockIdx.y;
    const float sh = MODE == 0 ? (noshift ? 0.f : (float)x[c * scs]) : mean[c];
    const float scl = MODE == 0 ? 1.f : invstd[c];
    float s0 = 0.f, s1 = 0.f;
    const int n_end = min(N, (g + 1) * npg);
    for (int n = g * npg; n < n_end; ++n)
        for (long s = threadIdx.x; s < HW; s += 256) {
            const long off = n * sn + c * scs + s * ss;
            if (MODE == 0) {
                const float dlt = (float)x[off] - sh;
                s0 += dlt;
                s1 += dlt * dlt;
            } else {
                float dz = (float)dout[off];
                if (relu && !((float)out[off] > 0.f)) dz = 0.f;
                s0 += dz;
                s1 += dz * (((float)x[off] - sh) * scl);
            }
        }
    s0 = wave_sum(s0);
    s1 = wave_sum(s1);
    __shared__ float w0[4], w1[4];
    if ((threadIdx.x & 63) == 0) {
        w0[threadIdx.x >> 6] = s0;
        w1[threadIdx.x >> 6] = s1;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        p0[(long)g * C + c] = (w0[0] + w0[1]) + (w0[2] + w0[3]);
        p1[(long)g * C + c] = (w1[0] + w1[1]) + (w1[2] + w1[3]);
    }
}

template <typename T, bool NCHW>
__global__ __launch_bounds__(256) void bn_apply_generic(const T *__restrict__ x, const T *__restrict__ res,
                                                        T *__restrict__ out, const float *__restrict__ scale,
                                                        const float *__restrict__ bias, long total, int C, long HW,
                                                        int relu)
{
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const int c = NCHW ? (int)((i / HW) % C) : (int)(i % C);
        float z = (float)x[i] * scale[c] + bias[c];
        if (res) z += (float)res[i];
        if (relu) z = z > 0.f ? z : 0.f;
        out[i] = (T)z;
    }
}

template <typename T, bool NCHW>
__global__ __launch_bounds__(256) void bn_bwd_apply_generic(const T *__restrict__ x, const T *__restrict__ out,
                                                            const T *__restrict__ dout, T *__restrict__ dx,
                                                            T *__restrict__ dres, const float *__restrict__ mean,
                                                            const float *__restrict__ invstd,
                                                            const float *__restrict__ coef, long total, int C,
                                                            long HW, int relu)
{
    const float *ca = coef, *cb = coef + C, *cc = coef + 2 * C;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const int c = NCHW ? (int)((i / HW) % C) : (int)(i % C);
        float dz = (float)dout[i];
        if (relu && !((float)out[i] > 0.f)) dz = 0.f;
        const float xhat = ((float)x[i] - mean[c]) * invstd[c];
        dx[i] = (T)(ca[c] * (dz - cb[c] - xhat * cc[c]));
        if (dres) dres[i] = (T)dz;
    }
}

// Folds many rows of partial sums into few: out[j][c] = sum of in[r][c] over the j-th run of `run` rows, for the
// two arrays (sums, sums of squares) that follow each other in both buffers.  Fixed order: reproducible.
__global__ __launch_bounds__(256) void bn_stats_fold(const float *__restrict__ in, int R, int C, int run,
                                                     float *__restrict__ out, int R2)
{
    const int j = blockIdx.x;
    const int r0 = j * run, r1 = min(R, r0 + run);
    for (int c = threadIdx.x; c < 2 * C; c += 256) {
        const int arr = c / C, cc = c - arr * C;
        const float *p = in + (size_t)arr * R * C + cc;
        float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
        int r = r0;
        for (; r + 3 < r1; r += 4) {
            s0 += p[(size_t)r * C];
            s1 += p[(size_t)(r + 1) * C];
            s2 += p[(size_t)(r + 2) * C];
            s3 += p[(size_t)(r + 3) * C];
        }
        for (; r < r1; ++r) s0 += p[(size_t)r * C];
        out[(size_t)arr * R2 * C + (size_t)j * C + cc] = (s0 + s1) + (s2 + s3);
    }
}

// ----------------------------------------------------------------------------- finalize (tiny)
// Column sums of the two arrays of partial sums for channel c, by one block of 256 threads: every thread adds the
// rows g = t, t + 256, ... (four independent loads at a time), then lanes and wavefronts are combined in a fixed
// order.  The result is valid in thread 0.
__device__ inline void block_column_sums(const float *__restrict__ p0, const float *__restrict__ p1, int G, int C, int c,
                                         double *S_out, double *Q_out)
{
    __shared__ double part[2][4];
    const int t = threadIdx.x;
    double S = 0.0, Q = 0.0;
    int g = t;
    for (; g + 768 < G; g += 1024) {
        const float a0 = p0[(long)g * C + c], a1 = p0[(long)(g + 256) * C + c], a2 = p0[(long)(g + 512) * C + c],
                    a3 = p0[(long)(g + 768) * C + c];
        const float b0 = p1[(long)g * C + c], b1 = p1[(long)(g + 256) * C + c], b2 = p1[(long)(g + 512) * C + c],
                    b3 = p1[(long)(g + 768) * C + c];
        S += ((double)a0 + (double)a1) + ((double)a2 + (double)a3);
        Q += ((double)b0 + (double)b1) + ((double)b2 + (double)b3);
    }
    for (; g < G; g += 256) {
        S += (double)p0[(long)g * C + c];
        Q += (double)p1[(long)g * C + c];
    }
    S = wave_sum_f64(S);
    Q = wave_sum_f64(Q);
    if ((t & 63) == 0) {
        part[0][t >> 6] = S;
        part[1][t >> 6] = Q;
    }
    __syncthreads();
    *S_out = (part[0][0] + part[0][1]) + (part[0][2] + part[0][3]);
    *Q_out = (part[1][0] + part[1][1]) + (part[1][2] + part[1][3]);
}

template <typename T>
__global__ __launch_bounds__(256) void bn_fwd_finalize(const float *__restrict__ p0, const float *__restrict__ p1, int G, int C, double M,
                                const T *__restrict__ x, long shift_stride, const float *__restrict__ gamma,
                                const float *__restrict__ beta, float eps, float momentum,
                                float *__restrict__ save_mean, float *__restrict__ save_invstd,
                                float *__restrict__ running_mean, float *__restrict__ running_var,
                                float *__restrict__ scale, float *__restrict__ bias)
{
    const int c = blockIdx.x;
    double S, Q;
    block_column_sums(p0, p1, G, C, c, &S, &Q);
    if (threadIdx.x != 0) return;
    const double ms = S / M;
    double var = Q / M - ms * ms;
    if (var < 0.0) var = 0.0;
    const double mean = (x ? (double)(float)x[c * shift_stride] : 0.0) + ms;   // x == nullptr: the sums are not shifted
    const double invstd = 1.0 / sqrt(var + (double)eps);
    save_mean[c] = (float)mean;
    save_invstd[c] = (float)invstd;
    const double sc = (double)gamma[c] * invstd;
    scale[c] = (float)sc;
    bias[c] = (float)((double)beta[c] - mean * sc);
    if (running_mean) {
        const double unbiased = M > 1.0 ? var * M / (M - 1.0) : var;
        running_mean[c] = (float)((1.0 - (double)momentum) * (double)running_mean[c] + (double)momentum * mean);
        running_var[c] = (float)((1.0 - (double)momentum) * (double)running_var[c] + (double)momentum * unbiased);
    }
}

__global__ __launch_bounds__(256) void bn_bwd_finalize(const float *__restrict__ p0, const float *__restrict__ p1, int G, int C, double M,
                                const float *__restrict__ gamma, const float *__restrict__ invstd,
                                float *__restrict__ dgamma, float *__restrict__ dbeta, float *__restrict__ coef)
{
    const int c = blockIdx.x;
    double S, Q;
    block_column_sums(p0, p1, G, C, c, &S, &Q);
    if (threadIdx.x != 0) return;
    dbeta[c] = (float)S;
    dgamma[c] = (float)Q;
    coef[c] = gamma[c] * invstd[c];
    coef[C + c] = (float)(S / M);
    coef[2 * C + c] = (float)(Q / M);
}

struct Geom {
    long M, HW, total;
    int G;
    bool fast;
    long rows_per_block;  // fast path
    int npg;              // generic path: images per partial block
    long sn, sc, ss;
};

Geom geometry(const nsk_bn_desc_t &d, bool backward)
{
    Geom g;
    g.HW = (long)d.H * d.W;
    g.M = (long)d.N * g.HW;
    g.total = g.M * d.C;
    g.fast = nhwc_fast(d);
    if (g.fast) {
        const int VEC = d.dtype == NSK_BF16 ? 8 : 4;
        const int RP = 256 / (d.C / VEC);
        // at least four passes of its 256 threads per block (measured on the 2-8 MB tensors of the CIFAR-sized network:
        // eight passes leave one block per CU there and the whole step 1.5% slower; two are no better than four)
        long G = (g.M + (long)RP * 4 - 1) / ((long)RP * 4);
        // Measured: the forward statistics pass over a large tensor (one input stream) is fastest with eight blocks
        // per CU, the backward pass (three input streams) and small tensors with two.
        // More blocks also mean more partial sums for the finalize kernel to read (G x C floats, twice): the larger
        // count is only used while that stays within 2 MB per array.
        long cap = (!backward && g.total >= (16L << 20)) ? 2048 : 512;
        if (cap * d.C > (512L << 10)) cap = 512;
        if (G > cap) G = cap;
        if (G < 1) G = 1;
        g.rows_per_block = (g.M + G - 1) / G;
        g.G = (int)((g.M + g.rows_per_block - 1) / g.rows_per_block);
        g.npg = 0;
    } else {
        int G = 1024 / d.C;
        if (G < 1) G = 1;
        if (G > d.N) G = d.N;
        g.npg = ceil_div(d.N, G);
        g.G = ceil_div(d.N, g.npg);
        g.rows_per_block = 0;
    }
    if (d.layout == NSK_NCHW) {
        g.sn = (long)d.C * g.HW;
        g.sc = g.HW;
        g.ss = 1;
    } else {
        g.sn = g.HW * d.C;
        g.sc = 1;
        g.ss = d.C;
    }
    return g;
}

int stream_blocks(long work_items)
{
    long b = (work_items + 255) / 256;
    const long cap = 256 * 16;  // 16 blocks per CU keep every CU streaming
    if (b > cap) b = cap;
    if (b < 1) b = 1;
    return (int)b;
}

template <typename T>
int bn_fwd_typed(const nsk_bn_desc_t &d, const T *x, const T *res, const float *gamma, const float *beta, T *out,
                 float *save_mean, float *save_invstd, float *running_mean, float *running_var, float *ws,
                 unsigned char *relu_mask, const float *stats, int stats_rows, hipStream_t stream)
{
    const Geom g = geometry(d, false);
    float *p0 = ws, *p1 = ws + (long)g.G * d.C, *scale = p1 + (long)g.G * d.C, *bias = scale + d.C;
    constexpr int VEC = BT<T>::VEC;
    if (stats) {
        // partial sums of x and x^2 left by the producer of x ([2][stats_rows][C], not shifted): no reduction pass.
        // A producer with small tiles leaves tens of thousands of rows: those are first folded into at most G rows
        // (the finalize kernel has one wavefront per channel).
        const float *q0 = stats, *q1 = stats + (long)stats_rows * d.C;
        int rows = stats_rows;
        if (stats_rows > 1024 && stats_rows > g.G) {
            const int run = ceil_div(stats_rows, g.G), r2 = ceil_div(stats_rows, run);
            hipLaunchKernelGGL(bn_stats_fold, dim3(r2), dim3(256), 0, stream, stats, stats_rows, d.C, run, p0, r2);
            q0 = p0;
            q1 = p0 + (long)r2 * d.C;
            rows = r2;
        }
        hipLaunchKernelGGL((bn_fwd_finalize<T>), dim3(d.C), dim3(256), 0, stream, q0, q1, rows, d.C,
                           (double)g.M, (const T *)nullptr, 0L, gamma, beta, d.eps, d.momentum, save_mean, save_invstd,
                           running_mean, running_var, scale, bias);
    } else if (g.fast) {
        hipLaunchKernelGGL((bn_reduce_nhwc<T, 0>), dim3(g.G), dim3(256), 0, stream, x, (const T *)nullptr,
                           (const T *)nullptr, (const float *)nullptr, (const float *)nullptr, 0, g.M, d.C,
                           g.rows_per_block, p0, p1, (unsigned char *)nullptr, (const unsigned char *)nullptr);
    } else {
        hipLaunchKernelGGL((bn_reduce_generic<T, 0>), dim3(d.C, g.G), dim3(256), 0, stream, x, (const T *)nullptr,
                           (const T *)nullptr, (const float *)nullptr, (const float *)nullptr, 0, d.N, g.HW, g.sn,
                           g.sc, g.ss, g.npg, d.C, p0, p1);
    }
    if (!stats)
        hipLaunchKernelGGL((bn_fwd_finalize<T>), dim3(d.C), dim3(256), 0, stream, p0, p1, g.G, d.C,
                           (double)g.M, x, g.sc, gamma, beta, d.eps, d.momentum, save_mean, save_invstd, running_mean,
                           running_var, scale, bias);
    if (g.fast) {
        const long nvec = g.total / VEC;
        const dim3 grid(stream_blocks(nvec));
#define NSK_APPLY(R, L) \
    hipLaunchKernelGGL((bn_apply_nhwc<T, R, L>), grid, dim3(256), 0, stream, x, res, out, scale, bias, nvec, d.C, relu_mask)
        if (res) {
            if (d.relu) NSK_APPLY(true, true); else NSK_APPLY(true, false);
        } else {
            if (d.relu) NSK_APPLY(false, true); else NSK_APPLY(false, false);
        }
#undef NSK_APPLY
    } else {
        const dim3 grid(stream_blocks(g.total));
        if (d.layout == NSK_NCHW)
            hipLaunchKernelGGL((bn_apply_generic<T, true>), grid, dim3(256), 0, stream, x, res, out, scale, bias,
                               g.total, d.C, g.HW, d.relu);
        else
            hipLaunchKernelGGL((bn_apply_generic<T, false>), grid, dim3(256), 0, stream, x, res, out, scale, bias,
                               g.total, d.C, g.HW, d.relu);
    }
    return check_launch();
}

template <typename T>
int bn_bwd_typed(const nsk_bn_desc_t &d, const T *x, const T *out, const T *dout, const float *gamma,
                 const float *mean, const float *invstd, T *dx, T *dres, float *dgamma, float *dbeta, float *ws,
                 const unsigned char *mask_in, hipStream_t stream, const float *act = nullptr)
{
    const Geom g = geometry(d, true);
    if (act && !(g.fast && d.relu)) return NSK_ERR_UNSUPPORTED;
    float *p0 = ws, *p1 = ws + (long)g.G * d.C, *coef = p1 + (long)g.G * d.C;
    // the ReLU mask bytes follow the float part of the workspace (see bn_mask_bytes)
    unsigned char *mask = (unsigned char *)ws + align_up((2 * (size_t)bn_partial_blocks(d) * d.C + 4 * (size_t)d.C) * sizeof(float));
    constexpr int VEC = BT<T>::VEC;
    if (g.fast) {
        hipLaunchKernelGGL((bn_reduce_nhwc<T, 1>), dim3(g.G), dim3(256), 0, stream, x, out, dout, mean, invstd,
                           d.relu, g.M, d.C, g.rows_per_block, p0, p1, mask, mask_in, 0, act);
    } else {
        hipLaunchKernelGGL((bn_reduce_generic<T, 1>), dim3(d.C, g.G), dim3(256), 0, stream, x, out, dout, mean,
                           invstd, d.relu, d.N, g.HW, g.sn, g.sc, g.ss, g.npg, d.C, p0, p1);
    }
    hipLaunchKernelGGL(bn_bwd_finalize, dim3(d.C), dim3(256), 0, stream, p0, p1, g.G, d.C,
                       (double)g.M, gamma, invstd, dgamma, dbeta, coef);
    if (g.fast) {
        const long nvec = g.total / VEC;
        const dim3 grid(stream_blocks(nvec));
#define NSK_BAPPLY(R, L)                                                                                       \
    hipLaunchKernelGGL((bn_bwd_apply_nhwc<T, R, L>), grid, dim3(256), 0, stream, x, out, dout, dx, dres, mean, \
                       invstd, coef, nvec, d.C, mask_in ? mask_in : mask)
        if (dres) {
            if (d.relu) NSK_BAPPLY(true, true); else NSK_BAPPLY(true, false);
        } else {
            if (d.relu) NSK_BAPPLY(false, true); else NSK_BAPPLY(false, false);
        }
#undef NSK_BAPPLY
    } else {
        const dim3 grid(stream_blocks(g.total));
        if (d.layout == NSK_NCHW)
            hipLaunchKernelGGL((bn_bwd_apply_generic<T, true>), grid, dim3(256), 0, stream, x, out, dout, dx, dres,
                               mean, invstd, coef, g.total, d.C, g.HW, d.relu);
        else
            hipLaunchKernelGGL((bn_bwd_apply_generic<T, false>), grid, dim3(256), 0, stream, x, out, dout, dx, dres,
                               mean, invstd, coef, g.total, d.C, g.HW, d.relu);
    }
    return check_launch();
}

}  // namespace

// Bytes of ReLU mask the backward pass keeps between its two kernels (one byte per 16-byte vector), 0 if unused.
size_t bn_mask_bytes(const nsk_bn_desc_t &d)
{
    if (!d.relu || !nhwc_fast(d)) return 0;
    const size_t vec = d.dtype == NSK_BF16 ? 8 : 4;
    return (size_t)d.N * d.H * d.W * d.C / vec;
}

int bn_partial_blocks(const nsk_bn_desc_t &d)
{
    const int f = geometry(d, false).G, b = geometry(d, true).G;
    return f > b ? f : b;
}

int launch_bn_fwd(const nsk_bn_desc_t &d, const void *x, const void *residual, const float *gamma,
                  const float *beta, void *out, float *save_mean, float *save_invstd, float *running_mean,
                  float *running_var, void *ws, unsigned char *relu_mask, const float *stats, int stats_rows,
                  hipStream_t stream)
{
    if (d.dtype == NSK_BF16)
        return bn_fwd_typed<bf16_t>(d, (const bf16_t *)x, (const bf16_t *)residual, gamma, beta, (bf16_t *)out,
                                    save_mean, save_invstd, running_mean, running_var, (float *)ws, relu_mask, stats,
                                    stats_rows, stream);
    return bn_fwd_typed<float>(d, (const float *)x, (const float *)residual, gamma, beta, (float *)out, save_mean,
                               save_invstd, running_mean, running_var, (float *)ws, relu_mask, stats, stats_rows, stream);
}

// Partial sums of x and x^2 per channel, [2][bn_stats_rows(d)][C] floats, not shifted: what the convolution kernels
// with a fused statistics epilogue write, produced here by a reduction pass for the shapes they do not cover.
int bn_stats_rows(const nsk_bn_desc_t &d) { return geometry(d, false).G; }

int launch_bn_stats(const nsk_bn_desc_t &d, const void *x, float *stats, hipStream_t stream)
{
    const Geom g = geometry(d, false);
    float *p0 = stats, *p1 = stats + (long)g.G * d.C;
#define NSK_STATS(T)                                                                                                   \
    if (g.fast)                                                                                                        \
        hipLaunchKernelGGL((bn_reduce_nhwc<T, 0>), dim3(g.G), dim3(256), 0, stream, (const T *)x, (const T *)nullptr,  \
                           (const T *)nullptr, (const float *)nullptr, (const float *)nullptr, 0, g.M, d.C,            \
                           g.rows_per_block, p0, p1, (unsigned char *)nullptr, (const unsigned char *)nullptr, 1);     \
    else                                                                                                               \
        hipLaunchKernelGGL((bn_reduce_generic<T, 0>), dim3(d.C, g.G), dim3(256), 0, stream, (const T *)x,              \
                           (const T *)nullptr, (const T *)nullptr, (const float *)nullptr, (const float *)nullptr, 0,  \
                           d.N, g.HW, g.sn, g.sc, g.ss, g.npg, d.C, p0, p1, 1)
    if (d.dtype == NSK_BF16) {
        NSK_STATS(bf16_t);
    } else {
        NSK_STATS(float);
    }
#undef NSK_STATS
    return check_launch();
}

int launch_bn_bwd(const nsk_bn_desc_t &d, const void *x, const void *out, const void *dout, const float *gamma,
                  const float *save_mean, const float *save_invstd, void *dx, void *dres, float *dgamma,
                  float *dbeta, void *ws, const unsigned char *relu_mask, hipStream_t stream, const float *act)
{
    if (d.dtype == NSK_BF16)
        return bn_bwd_typed<bf16_t>(d, (const bf16_t *)x, (const bf16_t *)out, (const bf16_t *)dout, gamma,
                                    save_mean, save_invstd, (bf16_t *)dx, (bf16_t *)dres, dgamma, dbeta,
                                    (float *)ws, relu_mask, stream, act);
    return bn_bwd_typed<float>(d, (const float *)x, (const float *)out, (const float *)dout, gamma, save_mean,
                               save_invstd, (float *)dx, (float *)dres, dgamma, dbeta, (float *)ws, relu_mask, stream, act);
}

// True if the fused-activation calls take this tensor: NHWC with a channel count the vector kernels handle.
bool bn_act_supported(const nsk_bn_desc_t &d) { return geometry(d, false).fast && geometry(d, true).fast; }

// Batch statistics and the coefficients of out = scale*x + shift (scale = gamma*invstd, shift = beta - mean*scale) from
// partial sums of x and x^2 ([2][stats_rows][C], not shifted), without the apply pass: coeffs = [2][C] floats.
int launch_bn_coeffs(const nsk_bn_desc_t &d, const float *gamma, const float *beta, const float *stats, int stats_rows,
                     float *save_mean, float *save_invstd, float *running_mean, float *running_var, float *coeffs,
                     void *ws, hipStream_t stream)
{
    const Geom g = geometry(d, false);
    float *p0 = (float *)ws;
    const float *q0 = stats, *q1 = stats + (long)stats_rows * d.C;
    int rows = stats_rows;
    if (stats_rows > 1024 && stats_rows > g.G) {
        const int run = ceil_div(stats_rows, g.G), r2 = ceil_div(stats_rows, run);
        hipLaunchKernelGGL(bn_stats_fold, dim3(r2), dim3(256), 0, stream, stats, stats_rows, d.C, run, p0, r2);
        q0 = p0;
        q1 = p0 + (long)r2 * d.C;
        rows = r2;
    }
    if (d.dtype == NSK_BF16)
        hipLaunchKernelGGL((bn_fwd_finalize<bf16_t>), dim3(d.C), dim3(256), 0, stream, q0, q1, rows, d.C, (double)g.M,
                           (const bf16_t *)nullptr, 0L, gamma, beta, d.eps, d.momentum, save_mean, save_invstd,
                           running_mean, running_var, coeffs, coeffs + d.C);
    else
        hipLaunchKernelGGL((bn_fwd_finalize<float>), dim3(d.C), dim3(256), 0, stream, q0, q1, rows, d.C, (double)g.M,
                           (const float *)nullptr, 0L, gamma, beta, d.eps, d.momentum, save_mean, save_invstd,
                           running_mean, running_var, coeffs, coeffs + d.C);
    return check_launch();
}

// out = relu(scale*x + shift) with the coefficients of launch_bn_coeffs: the apply pass on its own, for consumers
// whose kernel has no fused operand load.
int launch_bn_act(const nsk_bn_desc_t &d, const void *x, const float *coeffs, void *out, hipStream_t stream)
{
    const Geom g = geometry(d, false);
    if (!g.fast) return NSK_ERR_UNSUPPORTED;
    if (d.dtype == NSK_BF16) {
        const long nvec = g.total / BT<bf16_t>::VEC;
        hipLaunchKernelGGL((bn_apply_nhwc<bf16_t, false, true>), dim3(stream_blocks(nvec)), dim3(256), 0, stream, (const bf16_t *)x,
                           (const bf16_t *)nullptr, (bf16_t *)out, coeffs, coeffs + d.C, nvec, d.C, (unsigned char *)nullptr);
    } else {
        const long nvec = g.total / BT<float>::VEC;
        hipLaunchKernelGGL((bn_apply_nhwc<float, false, true>), dim3(stream_blocks(nvec)), dim3(256), 0, stream, (const float *)x,
                           (const float *)nullptr, (float *)out, coeffs, coeffs + d.C, nvec, d.C, (unsigned char *)nullptr);
    }
    return check_launch();
}

}  // namespace nsk

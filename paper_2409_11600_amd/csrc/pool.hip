// Max pooling forward / backward (the 3x3 stride-2 pool after the large-image stem of the ResNet
// recipe the paper follows, section "Experiments and Discussion").  Pure streaming: compares only.
// Forward records, per output, the window position r*S+s of the FIRST maximum in row-major order;
// backward is a gather over the (at most ceil(R/sh)*ceil(S/sw)) windows that contain an input
// element, so no atomics are needed and the result is reproducible.
#include <stdlib.h>

#include "nsk_internal.h"

namespace nsk {
namespace {

struct PoolGeom {
    int N, C, H, W, R, S, sh, sw, ph, pw, P, Q;
    long xs_n, xs_c, xs_h, xs_w;  // element strides of the input-shaped tensors
    long ys_n, ys_c, ys_h, ys_w;  // element strides of the output-shaped tensors
};

PoolGeom make_geom(const nsk_pool_desc_t &d, int P, int Q)
{
    PoolGeom g{d.N, d.C, d.H, d.W, d.R, d.S, d.stride_h, d.stride_w, d.pad_h, d.pad_w, P, Q, 0, 0, 0, 0, 0, 0, 0, 0};
    if (d.layout == NSK_NCHW) {
        g.xs_n = (long)d.C * d.H * d.W; g.xs_c = (long)d.H * d.W; g.xs_h = d.W; g.xs_w = 1;
        g.ys_n = (long)d.C * P * Q; g.ys_c = (long)P * Q; g.ys_h = Q; g.ys_w = 1;
    } else {
        g.xs_n = (long)d.H * d.W * d.C; g.xs_c = 1; g.xs_h = (long)d.W * d.C; g.xs_w = d.C;
        g.ys_n = (long)P * Q * d.C; g.ys_c = 1; g.ys_h = (long)Q * d.C; g.ys_w = d.C;
    }
    return g;
}

// One thread per (n, p, q, group of VEC channels).  VEC > 1 needs channel-contiguous (NHWC) data;
// with VEC = 1 the strides make it work for either layout (then consecutive threads walk the
// fastest-varying axis of the layout: c for NHWC, q for NCHW).
template <typename T, int VEC, bool NCHW>
__global__ __launch_bounds__(256) void maxpool_fwd_kernel(const T *__restrict__ x, T *__restrict__ y,
                                                          signed char *__restrict__ idx, const PoolGeom g)
{
    const int CV = g.C / VEC;
    const long total = (long)g.N * g.P * g.Q * CV;
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    int n, p, q, c;
    if (NCHW) {
        q = (int)(i % g.Q); long r = i / g.Q;
        p = (int)(r % g.P); r /= g.P;
        c = (int)(r % CV) * VEC; n = (int)(r / CV);
    } else {
        c = (int)(i % CV) * VEC; long r = i / CV;
        q = (int)(r % g.Q); r /= g.Q;
        p = (int)(r % g.P); n = (int)(r / g.P);
    }
    float best[VEC];
    int where[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        best[e] = -INFINITY;
        where[e] = -1;
    }
    for (int r = 0; r < g.R; ++r) {
        const int h = p * g.sh - g.ph + r;
        if ((unsigned)h >= (unsigned)g.H) continue;
        for (int s = 0; s < g.S; ++s) {
            const int w = q * g.sw - g.pw + s;
            if ((unsigned)w >= (unsigned)g.W) continue;
            const T *px = x + n * g.xs_n + c * g.xs_c + h * g.xs_h + w * g.xs_w;
            float v[VEC];
            if constexpr (VEC == 8) {
                const bf16x8 t = *(const bf16x8 *)px;
#pragma unroll
                for (int e = 0; e < VEC; ++e) v[e] = (float)t[e];
            } else if constexpr (VEC == 4) {
                const f32x4 t = *(const f32x4 *)px;
#pragma unroll
                for (int e = 0; e < VEC; ++e) v[e] = t[e];
            } else {
                v[0] = (float)px[0];
            }
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const float f = v[e];
                if (where[e] < 0 || f > best[e]) {
                    best[e] = f;
                    where[e] = r * g.S + s;
                }
            }
        }
    }
    const long o = n * g.ys_n + c * g.ys_c + p * g.ys_h + q * g.ys_w;
    if constexpr (VEC == 8) {
        bf16x8 yv;
        unsigned long long iv = 0;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            yv[e] = (bf16_t)best[e];
            iv |= (unsigned long long)(unsigned char)(signed char)where[e] << (8 * e);
        }
        *(bf16x8 *)(y + o) = yv;
        *(unsigned long long *)(idx + o) = iv;
    } else if constexpr (VEC == 4) {
        f32x4 yv;
        unsigned iv = 0;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            yv[e] = best[e];
            iv |= (unsigned)(unsigned char)(signed char)where[e] << (8 * e);
        }
        *(f32x4 *)(y + o) = yv;
        *(unsigned *)(idx + o) = iv;
    } else {
        y[o] = (T)best[0];
        idx[o] = (signed char)where[0];
    }
}

// 3x3 windows on vectorised NHWC tensors (the pool of the large-image stem): the nine loads of a lane go through a
// buffer descriptor (an offset of ~0 is out of range: no branch per tap), so they are all in flight before the first
// comparison; the comparisons run in the same order as in the general kernel (first maximum wins, padding never does).
template <typename T, int VEC>
__global__ __launch_bounds__(256) void maxpool3_fwd_nhwc_kernel(const T *__restrict__ x, T *__restrict__ y,
                                                                signed char *__restrict__ idx, const PoolGeom g,
                                                                const unsigned x_bytes)
{
    typedef T Vec __attribute__((ext_vector_type(VEC)));
    static_assert(sizeof(Vec) == 16, "one 16-byte load per tap");
    const int CV = g.C / VEC;
    const long total = (long)g.N * g.P * g.Q * CV;
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int c = (int)(i % CV) * VEC;
    long r_ = i / CV;
    const int q = (int)(r_ % g.Q);
    r_ /= g.Q;
    const int p = (int)(r_ % g.P), n = (int)(r_ / g.P);
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)x, 0, x_bytes, 0x00020000);
    const int h0 = p * g.sh - g.ph, w0 = q * g.sw - g.pw;
    Vec v[9];
    bool ok[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        const int h = h0 + t / 3, w = w0 + t % 3;
        ok[t] = (unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W;
        const unsigned off = (unsigned)(((((long)n * g.H + h) * g.W + w) * g.C + c) * (long)sizeof(T));
        v[t] = __builtin_bit_cast(Vec, __builtin_amdgcn_raw_buffer_load_b128(rsrc, ok[t] ? off : ~0u, 0, 0));
    }
    float best[VEC];
    int where[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        best[e] = -INFINITY;
        where[e] = -1;
    }
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        if (!ok[t]) continue;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const float f = (float)v[t][e];
            if (where[e] < 0 || f > best[e]) {
                best[e] = f;
                where[e] = t;
            }
        }
    }
    const long o = (((long)n * g.P + p) * g.Q + q) * g.C + c;
    Vec yv;
#pragma unroll
    for (int e = 0; e < VEC; ++e) yv[e] = (T)best[e];
    __builtin_nontemporal_store(yv, (Vec *)(y + o));
    if constexpr (VEC == 8) {
        unsigned long long iv = 0;
#pragma unroll
        for (int e = 0; e < VEC; ++e) iv |= (unsigned long long)(unsigned char)(signed char)where[e] << (8 * e);
        __builtin_nontemporal_store(iv, (unsigned long long *)(idx + o));
    } else {
        unsigned iv = 0;
#pragma unroll
        for (int e = 0; e < VEC; ++e) iv |= (unsigned)(unsigned char)(signed char)where[e] << (8 * e);
        __builtin_nontemporal_store(iv, (unsigned *)(idx + o));
    }
}

template <typename T, int VEC, bool NCHW>
__global__ __launch_bounds__(256) void maxpool_bwd_kernel(const T *__restrict__ dy, const signed char *__restrict__ idx,
                                                          T *__restrict__ dx, const PoolGeom g)
{
    const int CV = g.C / VEC;
    const long total = (long)g.N * g.H * g.W * CV;
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    int n, h, w, c;
    if (NCHW) {
        w = (int)(i % g.W); long r = i / g.W;
        h = (int)(r % g.H); r /= g.H;
        c = (int)(r % CV) * VEC; n = (int)(r / CV);
    } else {
        c = (int)(i % CV) * VEC; long r = i / CV;
        w = (int)(r % g.W); r /= g.W;
        h = (int)(r % g.H); n = (int)(r / g.H);
    }
    float acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
    // windows p with p*sh - ph <= h <= p*sh - ph + R - 1
    int p_lo = h + g.ph - g.R + 1;
    p_lo = p_lo <= 0 ? 0 : (p_lo + g.sh - 1) / g.sh;
    int p_hi = (h + g.ph) / g.sh;
    if (p_hi > g.P - 1) p_hi = g.P - 1;
    int q_lo = w + g.pw - g.S + 1;
    q_lo = q_lo <= 0 ? 0 : (q_lo + g.sw - 1) / g.sw;
    int q_hi = (w + g.pw) / g.sw;
    if (q_hi > g.Q - 1) q_hi = g.Q - 1;
    for (int p = p_lo; p <= p_hi; ++p)
        for (int q = q_lo; q <= q_hi; ++q) {
            const int pos = (h + g.ph - p * g.sh) * g.S + (w + g.pw - q * g.sw);
            const long o = n * g.ys_n + c * g.ys_c + p * g.ys_h + q * g.ys_w;
            if constexpr (VEC == 8) {   // one 8-byte index load and one 16-byte gradient load per window
                const unsigned long long iv = *(const unsigned long long *)(idx + o);
                const bf16x8 gv = *(const bf16x8 *)(dy + o);
#pragma unroll
                for (int e = 0; e < VEC; ++e)
                    if ((int)(signed char)(iv >> (8 * e)) == pos) acc[e] += (float)gv[e];
            } else if constexpr (VEC == 4) {
                const unsigned iv = *(const unsigned *)(idx + o);
                const f32x4 gv = *(const f32x4 *)(dy + o);
#pragma unroll
                for (int e = 0; e < VEC; ++e)
                    if ((int)(signed char)(iv >> (8 * e)) == pos) acc[e] += gv[e];
            } else {
                if (idx[o] == pos) acc[0] += (float)dy[o];
            }
        }
    const long o = n * g.xs_n + c * g.xs_c + h * g.xs_h + w * g.xs_w;
    if constexpr (VEC == 8) {
        bf16x8 v;
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] = (bf16_t)acc[e];
        *(bf16x8 *)(dx + o) = v;
    } else if constexpr (VEC == 4) {
        f32x4 v;
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] = acc[e];
        *(f32x4 *)(dx + o) = v;
    } else {
        dx[o] = (T)acc[0];
    }
}

// Backward of the 3x3 stride-2 pad-1 pool on even H, W (the stem's pool), channel-contiguous data: one thread per
// 2x2 block of input pixels and VEC channels.  The block (rows 2m, 2m+1, columns 2n, 2n+1) lies in the windows
// p in {m, m+1}, q in {n, n+1} only, so four window loads serve four pixels (the per-pixel kernel needs nine).
// Window (p, q) covers rows 2p-1..2p+1: row 2m is its row r = 1 for p = m; row 2m+1 is r = 2 for p = m and r = 0
// for p = m+1; columns likewise.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void maxpool3s2_bwd_kernel(const T *__restrict__ dy, const signed char *__restrict__ idx,
                                                             T *__restrict__ dx, int N, int C, int H, int W)
{
    typedef T Vec __attribute__((ext_vector_type(VEC)));
    const int CV = C / VEC, P = H / 2, Q = W / 2;
    const long total = (long)N * P * Q * CV;
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int c = (int)(i % CV) * VEC;
    long r = i / CV;
    const int n_ = (int)(r % Q);
    r /= Q;
    const int m = (int)(r % P), img = (int)(r / P);
    float acc[2][2][VEC];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[a][b][e] = 0.f;
#pragma unroll
    for (int dp = 0; dp < 2; ++dp)
#pragma unroll
        for (int dq = 0; dq < 2; ++dq) {
            const int p = m + dp, q = n_ + dq;
            if (p >= P || q >= Q) continue;
            const long o = (((long)img * P + p) * Q + q) * C + c;
            Vec gv;
            unsigned long long iv;
            if constexpr (VEC == 8) {
                iv = __builtin_nontemporal_load((const unsigned long long *)(idx + o));
            } else {
                iv = __builtin_nontemporal_load((const unsigned *)(idx + o));
            }
            gv = __builtin_nontemporal_load((const Vec *)(dy + o));
            // pixel (a, b) of the block is window position (ra, sb) of window (p, q), if it is inside it
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                const int ra = dp == 0 ? a + 1 : (a == 1 ? 0 : -1);
                if (ra < 0) continue;
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    const int sb = dq == 0 ? b + 1 : (b == 1 ? 0 : -1);
                    if (sb < 0) continue;
                    const int pos = ra * 3 + sb;
#pragma unroll
                    for (int e = 0; e < VEC; ++e)
                        if ((int)(signed char)(iv >> (8 * e)) == pos) acc[a][b][e] += (float)gv[e];
                }
            }
        }
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            Vec v;
#pragma unroll
            for (int e = 0; e < VEC; ++e) v[e] = (T)acc[a][b][e];
            __builtin_nontemporal_store(v, (Vec *)(dx + ((((long)img * H + 2 * m + a) * W + 2 * n_ + b) * C + c)));
        }
}

template <typename T, int VEC>
int pool_typed(bool fwd, const nsk_pool_desc_t &d, int P, int Q, const void *a, void *b, const signed char *idx_in,
               signed char *idx_out, hipStream_t stream)
{
    const PoolGeom g = make_geom(d, P, Q);
    const bool vec = d.layout == NSK_NHWC && d.C % VEC == 0;
    if (!fwd && vec && d.R == 3 && d.S == 3 && d.stride_h == 2 && d.stride_w == 2 && d.pad_h == 1 && d.pad_w == 1 &&
        d.H % 2 == 0 && d.W % 2 == 0) {
        const long blocks2 = (long)d.N * (d.H / 2) * (d.W / 2) * (d.C / VEC);
        if (blocks2 == 0) return NSK_OK;
        hipLaunchKernelGGL((maxpool3s2_bwd_kernel<T, VEC>), dim3((unsigned)((blocks2 + 255) / 256)), dim3(256), 0, stream,
                           (const T *)a, idx_in, (T *)b, d.N, d.C, d.H, d.W);
        return check_launch();
    }
    const long pix = fwd ? (long)d.N * P * Q : (long)d.N * d.H * d.W;
    const long total = pix * (vec ? d.C / VEC : d.C);
    if (total == 0) return NSK_OK;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (fwd) {
        const unsigned long long x_bytes = (unsigned long long)d.N * d.H * d.W * d.C * sizeof(T);
        if (vec && d.R == 3 && d.S == 3 && x_bytes < 0xF0000000ull && !hooks().pool_general)   // (test hook)
            hipLaunchKernelGGL((maxpool3_fwd_nhwc_kernel<T, VEC>), grid, block, 0, stream, (const T *)a, (T *)b, idx_out, g,
                               (unsigned)x_bytes);
        else if (vec)
            hipLaunchKernelGGL((maxpool_fwd_kernel<T, VEC, false>), grid, block, 0, stream, (const T *)a, (T *)b, idx_out, g);
        else if (d.layout == NSK_NCHW)
            hipLaunchKernelGGL((maxpool_fwd_kernel<T, 1, true>), grid, block, 0, stream, (const T *)a, (T *)b, idx_out, g);
        else
            hipLaunchKernelGGL((maxpool_fwd_kernel<T, 1, false>), grid, block, 0, stream, (const T *)a, (T *)b, idx_out, g);
    } else {
        if (vec)
            hipLaunchKernelGGL((maxpool_bwd_kernel<T, VEC, false>), grid, block, 0, stream, (const T *)a, idx_in, (T *)b, g);
        else if (d.layout == NSK_NCHW)
            hipLaunchKernelGGL((maxpool_bwd_kernel<T, 1, true>), grid, block, 0, stream, (const T *)a, idx_in, (T *)b, g);
        else
            hipLaunchKernelGGL((maxpool_bwd_kernel<T, 1, false>), grid, block, 0, stream, (const T *)a, idx_in, (T *)b, g);
    }
    return check_launch();
}

}  // namespace

int launch_maxpool_fwd(const nsk_pool_desc_t &d, int P, int Q, const void *x, void *y, signed char *idx,
                       hipStream_t stream)
{
    if (d.dtype == NSK_BF16) return pool_typed<bf16_t, 8>(true, d, P, Q, x, y, nullptr, idx, stream);
    return pool_typed<float, 4>(true, d, P, Q, x, y, nullptr, idx, stream);
}

int launch_maxpool_bwd(const nsk_pool_desc_t &d, int P, int Q, const void *dy, const signed char *idx, void *dx,
                       hipStream_t stream)
{
    if (d.dtype == NSK_BF16) return pool_typed<bf16_t, 8>(false, d, P, Q, dy, dx, idx, nullptr, stream);
    return pool_typed<float, 4>(false, d, P, Q, dy, dx, idx, nullptr, stream);
}

}  // namespace nsk

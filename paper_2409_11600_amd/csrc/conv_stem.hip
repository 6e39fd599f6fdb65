// The image stem: a stride-2 convolution with very few input channels (7x7 stride 2 pad 3, 3 -> 64 on
// 224 x 224 inputs in the large-image recipe the paper follows, section "Experiments and Discussion").
//
// With 3 channels a filter tap is 6 bytes: nothing can be fetched with 16-byte loads and the reduction
// index (147) does not tile the MFMA k-step.  The stem is therefore rewritten as a stride-1 convolution
// on a SPACE-TO-DEPTH copy of the image:
//     x2[n][i][j][(a,b,c)] = x[n][2i+a][2j+b][c],  a,b in {0,1}, channels padded with zeros to 16
// A filter row r - pad = 2u + a splits into a coarse tap u and a phase a, so
//     y[n,p,q,k] = sum_{u,v,(a,b,c)} x2[n, p+u, q+v, (a,b,c)] * w2[k][u,v][(a,b,c)]
// with w2[k][u,v][(a,b,c)] = w[k][2u+a+pad][2v+b+pad][c] (zero where that tap does not exist).  A 7x7
// stride-2 filter becomes a 4x4 stride-1 filter over 16 channels: 256 reduction elements instead of
// 147 (1.74x the multiplies), but every pass now runs on the vectorised MFMA kernels:
//   forward        implicit GEMM on x2 (16 taps x 16 channels),
//   backward-weight the split-K kernel on x2, then dw2 is folded back into dw's layout,
//   backward-data  implicit GEMM producing dx2 (16 "channels" = the 2x2 phases x C), then depth-to-space.
// The bf16 7x7 stem with 64 output channels takes the halo kernels of conv_stem_halo.hip for the two GEMMs.
// The copies (x -> x2, dx2 -> dx) are plain streaming passes over the small 3-channel image.
#include "nsk_internal.h"

namespace nsk {
namespace {

constexpr int SC = 16;   // channels of the space-to-depth image

struct StemGeo {
    int N, C, H, W, K, R, pad, U, umin, H2, W2;
    int dtype;
    size_t es;
};

StemGeo stem_geo(const ConvGeo &g)
{
    StemGeo s;
    s.N = g.N; s.C = g.C; s.H = g.H; s.W = g.W; s.K = g.K; s.R = g.R; s.pad = g.ph;
    // r - pad = 2u + a: u from floor(-pad/2) to floor((R-1-pad)/2)
    s.umin = -((g.ph + 1) / 2);
    const int umax = (g.R - 1 - g.ph) >= 0 ? (g.R - 1 - g.ph) / 2 : -((g.ph - g.R + 2) / 2);
    s.U = umax - s.umin + 1;
    s.H2 = g.H / 2; s.W2 = g.W / 2;
    s.dtype = g.dtype; s.es = g.es;
    return s;
}

// Element strides of an image tensor in either layout.
struct ImgStrides {
    long n, c, h, w;
};

ImgStrides img_strides(int layout, int C, int H, int W)
{
    if (layout == NSK_NCHW) return {(long)C * H * W, (long)H * W, (long)W, 1L};
    return {(long)H * W * C, 1L, (long)W * C, (long)C};
}

// x (either layout, CC <= 4 channels) -> x2 (N, H/2, W/2, 16) NHWC: one thread per coarse pixel
template <typename T, int CC>
__global__ __launch_bounds__(256) void s2d_kernel(const T *__restrict__ x, T *__restrict__ x2, long total, int H, int W,
                                                  const ImgStrides xs)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int W2 = W / 2, H2 = H / 2;
    const int j = (int)(i % W2);
    const long r = i / W2;
    const int ii = (int)(r % H2);
    const long n = r / H2;
    typedef T vec_t __attribute__((ext_vector_type(SC)));
    vec_t o;
#pragma unroll
    for (int e = 0; e < SC; ++e) o[e] = (T)0.f;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const T *p = x + n * xs.n + (2 * ii + a) * xs.h + (2 * j + b) * xs.w;
#pragma unroll
            for (int c = 0; c < CC; ++c) o[(a * 2 + b) * CC + c] = p[c * xs.c];
        }
    *(vec_t *)(x2 + i * SC) = o;
}

// dx (either layout, CC <= 4 channels) (=|+=) depth-to-space of dx2 (N, H/2, W/2, 16)
template <typename T, int CC>
__global__ __launch_bounds__(256) void d2s_kernel(const T *__restrict__ dx2, T *__restrict__ dx, long total, int H, int W,
                                                  const ImgStrides xs, int accumulate)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int W2 = W / 2, H2 = H / 2;
    const int j = (int)(i % W2);
    const long r = i / W2;
    const int ii = (int)(r % H2);
    const long n = r / H2;
    typedef T vec_t __attribute__((ext_vector_type(SC)));
    const vec_t s = *(const vec_t *)(dx2 + i * SC);
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            T *p = dx + n * xs.n + (2 * ii + a) * xs.h + (2 * j + b) * xs.w;
#pragma unroll
            for (int c = 0; c < CC; ++c) {
                float v = (float)s[(a * 2 + b) * CC + c];
                if (accumulate) v += (float)p[c * xs.c];
                p[c * xs.c] = (T)v;
            }
        }
}

// Filter in either layout (element (k,c,r,s) at k*sk + c*sc + r*sr + s*ss) -> packed for the x2 problem.
//   MODE 0 (fwd):   out[k][u*U+v][(a,b,c)]           rows = output channel
//   MODE 1 (dgrad): out[(a,b,c)][u*U+v][k]           rows = phase-channel of dx2
template <typename T, int MODE>
__global__ __launch_bounds__(256) void stem_pack_kernel(const T *__restrict__ w, T *__restrict__ out, int K, int C, int R, int pad,
                                                        int U, int umin, long sk, long sc, long sr, long ss)
{
    const int total = K * U * U * SC;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    int k, t, e;
    if (MODE == 0) {
        e = i % SC; t = (i / SC) % (U * U); k = i / (SC * U * U);
    } else {
        k = i % K; t = (i / K) % (U * U); e = i / (K * U * U);
    }
    const int u = t / U + umin, v = t % U + umin;
    T val = (T)0.f;
    if (e < 4 * C) {
        const int c = e % C, ab = e / C, a = ab >> 1, b = ab & 1;
        const int r = 2 * u + a + pad, s = 2 * v + b + pad;
        if (r >= 0 && r < R && s >= 0 && s < R) val = w[k * sk + c * sc + r * sr + s * ss];
    }
    out[i] = val;
}

// dw (float, element (k,c,r,s) at k*sk + c*sc + r*sr + s*ss) (=|+=) dw2[k][u*U+v][(a,b,c)]
__global__ __launch_bounds__(256) void stem_unpack_dw_kernel(const float *__restrict__ dw2, float *__restrict__ dw, int K, int C, int R,
                                                             int pad, int U, int umin, long sk, long sc, long sr, long ss,
                                                             int accumulate)
{
    const int total = K * C * R * R;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int s = i % R, r = (i / R) % R, c = (i / (R * R)) % C, k = i / (R * R * C);
    // r - pad = 2u + a with a in {0,1}
    const int dr = r - pad, ds = s - pad;
    const int a = dr & 1, b = ds & 1;
    const int u = (dr - a) / 2 - umin, v = (ds - b) / 2 - umin;
    const float g = dw2[((long)k * U * U + u * U + v) * SC + (a * 2 + b) * C + c];
    float *o = dw + k * sk + c * sc + r * sr + s * ss;
    *o = accumulate ? *o + g : g;
}

struct StemPlan {
    size_t x2 = 0, w2 = 0, dx2 = 0, act = 0, part = 0, dw2 = 0, total = 0;
    int splits = 1, rows_per_split = 0;
    bool wide = false;   // backward-weight through the large-tile kernel
};

// backward-weight on the space-to-depth image: 16 channels, stride 1, U x U taps
void stem_wgrad_geometry(const ConvGeo &g, const StemGeo &s, WgradArgs *a)
{
    a->Nimg = s.N; a->H = s.H2; a->W = s.W2; a->C = SC; a->P = g.P; a->Q = g.Q; a->K = s.K;
    a->sh = 1; a->sw = 1; a->ph = -s.umin; a->pw = -s.umin;
    a->ntaps = s.U * s.U;
    a->L = s.N * g.P * g.Q;
    for (int t = 0; t < a->ntaps; ++t) {
        a->off_h[t] = (short)(t / s.U);
        a->off_w[t] = (short)(t % s.U);
    }
}

StemPlan stem_plan(const ConvGeo &g, const StemGeo &s, int pass)
{
    StemPlan p;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += align_up(bytes);
        return at;
    };
    const bool nchw = g.layout == NSK_NCHW;
    const size_t img2 = (size_t)s.N * s.H2 * s.W2 * SC * s.es;
    const size_t w2 = (size_t)s.K * s.U * s.U * SC;
    if (pass == NSK_PASS_FWD) {
        p.x2 = take(img2);
        p.w2 = take(w2 * s.es);
        if (nchw) p.act = take(g.y_elems * g.es);   // NHWC result before conversion
    } else if (pass == NSK_PASS_DGRAD) {
        p.w2 = take(w2 * s.es);
        p.dx2 = take(img2);
        if (nchw) p.act = take(g.y_elems * g.es);   // NHWC copy of dy
    } else {
        p.x2 = take(img2);
        if (nchw) p.act = take(g.y_elems * g.es);   // NHWC copy of dy
        WgradArgs wa{};
        stem_wgrad_geometry(g, s, &wa);
        p.wide = wgrad_wide_applicable(s.dtype, wa);
        p.rows_per_split = p.wide ? wgrad_wide_rows_per_split(wa, &p.splits)
                                  : wgrad_rows_per_split(s.dtype, wa.L, s.K, s.U * s.U * SC, &p.splits);
        p.part = take((size_t)p.splits * w2 * sizeof(float));
        p.dw2 = take(w2 * sizeof(float));
    }
    p.total = off;
    return p;
}

void filter_strides(const ConvGeo &g, long *sk, long *sc, long *sr, long *ss)
{
    if (g.layout == NSK_NCHW) {   // KCRS
        *sk = (long)g.C * g.R * g.S; *sc = (long)g.R * g.S; *sr = g.S; *ss = 1;
    } else {                      // KRSC
        *sk = (long)g.R * g.S * g.C; *sr = (long)g.S * g.C; *ss = g.C; *sc = 1;
    }
}

template <typename T, int CC>
int s2d_cc(const ConvGeo &g, const StemGeo &s, const void *x, void *x2, hipStream_t st)
{
    const long total = (long)s.N * s.H2 * s.W2;
    hipLaunchKernelGGL((s2d_kernel<T, CC>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const T *)x, (T *)x2, total,
                       s.H, s.W, img_strides(g.layout, s.C, s.H, s.W));
    return check_launch();
}

template <typename T>
int s2d_typed(const ConvGeo &g, const StemGeo &s, const void *x, void *x2, hipStream_t st)
{
    switch (s.C) {
    case 1: return s2d_cc<T, 1>(g, s, x, x2, st);
    case 2: return s2d_cc<T, 2>(g, s, x, x2, st);
    case 3: return s2d_cc<T, 3>(g, s, x, x2, st);
    default: return s2d_cc<T, 4>(g, s, x, x2, st);
    }
}

int space_to_depth(const ConvGeo &g, const StemGeo &s, const void *x, void *x2, hipStream_t st)
{
    return s.dtype == NSK_BF16 ? s2d_typed<bf16_t>(g, s, x, x2, st) : s2d_typed<float>(g, s, x, x2, st);
}

template <typename T, int CC>
int d2s_cc(const ConvGeo &g, const StemGeo &s, const void *dx2, void *dx, int accumulate, hipStream_t st)
{
    const long total = (long)s.N * s.H2 * s.W2;
    hipLaunchKernelGGL((d2s_kernel<T, CC>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const T *)dx2, (T *)dx, total,
                       s.H, s.W, img_strides(g.layout, s.C, s.H, s.W), accumulate);
    return check_launch();
}

template <typename T>
int d2s_typed(const ConvGeo &g, const StemGeo &s, const void *dx2, void *dx, int accumulate, hipStream_t st)
{
    switch (s.C) {
    case 1: return d2s_cc<T, 1>(g, s, dx2, dx, accumulate, st);
    case 2: return d2s_cc<T, 2>(g, s, dx2, dx, accumulate, st);
    case 3: return d2s_cc<T, 3>(g, s, dx2, dx, accumulate, st);
    default: return d2s_cc<T, 4>(g, s, dx2, dx, accumulate, st);
    }
}

template <int MODE>
int pack_filter(const ConvGeo &g, const StemGeo &s, const void *w, void *w2, hipStream_t st)
{
    long sk, sc, sr, ss;
    filter_strides(g, &sk, &sc, &sr, &ss);
    const int total = s.K * s.U * s.U * SC;
    if (s.dtype == NSK_BF16)
        hipLaunchKernelGGL((stem_pack_kernel<bf16_t, MODE>), dim3((total + 255) / 256), dim3(256), 0, st, (const bf16_t *)w,
                           (bf16_t *)w2, s.K, s.C, s.R, s.pad, s.U, s.umin, sk, sc, sr, ss);
    else
        hipLaunchKernelGGL((stem_pack_kernel<float, MODE>), dim3((total + 255) / 256), dim3(256), 0, st, (const float *)w,
                           (float *)w2, s.K, s.C, s.R, s.pad, s.U, s.umin, sk, sc, sr, ss);
    return check_launch();
}

#define STEM_TRY(expr)                \
    do {                              \
        const int st__ = (expr);      \
        if (st__ != NSK_OK) return st__; \
    } while (0)

}  // namespace

bool stem_applicable(const ConvGeo &g)
{
    if (g.sh != 2 || g.sw != 2 || g.dh != 1 || g.dw != 1) return false;
    if (g.C > 4 || g.R != g.S || g.R % 2 == 0 || g.R > 7) return false;
    if (g.ph != (g.R - 1) / 2 || g.pw != g.ph) return false;
    if (g.H % 2 || g.W % 2) return false;
    return !hooks().no_stem;
}

size_t stem_workspace_bytes(const ConvGeo &g, int pass) { return stem_plan(g, stem_geo(g), pass).total; }

int stem_stats_rows(const ConvGeo &g)
{
    const StemGeo s = stem_geo(g);
    return stem_halo_applicable(s.dtype, s.U, s.K, s.N, s.H2, s.W2) ? stem_halo_stats_rows(s.N, s.H2, s.W2) : 0;
}

int stem_fwd(const ConvGeo &g, const void *x, const void *w, void *y, char *ws, float *stats, int stats_rows, void **y_nhwc,
             hipStream_t st)
{

    const StemGeo s = stem_geo(g);
    const StemPlan p = stem_plan(g, s, NSK_PASS_FWD);
    const bool nchw = g.layout == NSK_NCHW;
    STEM_TRY(space_to_depth(g, s, x, ws + p.x2, st));
    STEM_TRY(pack_filter<0>(g, s, w, ws + p.w2, st));
    void *dst = nchw ? (void *)(ws + p.act) : y;
    if (y_nhwc) *y_nhwc = dst;
    if (stem_halo_applicable(s.dtype, s.U, s.K, s.N, s.H2, s.W2)) {
        STEM_TRY(launch_stem_halo(0, ws + p.x2, ws + p.w2, dst, s.N, s.H2, s.W2, stats, stats_rows, st));
        if (nchw) STEM_TRY(launch_nhwc_to_nchw(g.dtype, dst, y, g.N, g.K, g.P, g.Q, 0, st));
        return NSK_OK;
    }
    IgemmArgs a{};
    a.src = ws + p.x2; a.wpk = ws + p.w2; a.out = dst;
    a.Nimg = s.N; a.Hs = s.H2; a.Ws = s.W2; a.Cs = SC;
    a.Mi = g.P; a.Mj = g.Q; a.M = s.N * g.P * g.Q;
    a.mult_h = 1; a.add_h = s.umin; a.mult_w = 1; a.add_w = s.umin;
    a.ntaps = s.U * s.U; a.Ktot = a.ntaps * SC;
    a.Ngemm = s.K;
    a.Ho = g.P; a.Wo = g.Q; a.Co = s.K; a.osh = 1; a.oa = 0; a.osw = 1; a.ob = 0;
    a.accumulate = 0;
    a.src_bytes = (unsigned)((size_t)s.N * s.H2 * s.W2 * SC * s.es);
    a.wpk_bytes = (unsigned)((size_t)s.K * a.ntaps * SC * s.es);
    for (int t = 0; t < a.ntaps; ++t) {
        a.off_h[t] = (short)(t / s.U);
        a.off_w[t] = (short)(t % s.U);
    }
    STEM_TRY(launch_igemm(s.dtype, a, st));
    if (nchw) STEM_TRY(launch_nhwc_to_nchw(g.dtype, dst, y, g.N, g.K, g.P, g.Q, 0, st));
    return NSK_OK;
}

int stem_dgrad(const ConvGeo &g, const void *dy, const void *w, void *dx, int accumulate, char *ws, hipStream_t st)
{
    const StemGeo s = stem_geo(g);
    const StemPlan p = stem_plan(g, s, NSK_PASS_DGRAD);
    const void *src = dy;
    if (g.layout == NSK_NCHW) {
        STEM_TRY(launch_nchw_to_nhwc(g.dtype, dy, ws + p.act, g.N, g.K, g.P, g.Q, st));
        src = ws + p.act;
    }
    STEM_TRY(pack_filter<1>(g, s, w, ws + p.w2, st));
    // dx2[n,i,j,e] = sum_{u,v,k} dy[n, i-u, j-v, k] * w2[k][u,v][e]
    if (stem_halo_applicable(s.dtype, s.U, s.K, s.N, s.H2, s.W2)) {
        STEM_TRY(launch_stem_halo(1, src, ws + p.w2, ws + p.dx2, s.N, s.H2, s.W2, nullptr, 0, st));
        return s.dtype == NSK_BF16 ? d2s_typed<bf16_t>(g, s, ws + p.dx2, dx, accumulate, st)
                                   : d2s_typed<float>(g, s, ws + p.dx2, dx, accumulate, st);
    }
    IgemmArgs a{};
    a.src = src; a.wpk = ws + p.w2; a.out = ws + p.dx2;
    a.Nimg = s.N; a.Hs = g.P; a.Ws = g.Q; a.Cs = s.K;
    a.Mi = s.H2; a.Mj = s.W2; a.M = s.N * s.H2 * s.W2;
    a.mult_h = 1; a.add_h = 0; a.mult_w = 1; a.add_w = 0;
    a.ntaps = s.U * s.U; a.Ktot = a.ntaps * s.K;
    a.Ngemm = SC;
    a.Ho = s.H2; a.Wo = s.W2; a.Co = SC; a.osh = 1; a.oa = 0; a.osw = 1; a.ob = 0;
    a.accumulate = 0;
    a.src_bytes = (unsigned)(g.y_elems * s.es);
    a.wpk_bytes = (unsigned)((size_t)s.K * a.ntaps * SC * s.es);
    for (int t = 0; t < a.ntaps; ++t) {
        a.off_h[t] = (short)(-(t / s.U + s.umin));
        a.off_w[t] = (short)(-(t % s.U + s.umin));
    }
    STEM_TRY(launch_igemm(s.dtype, a, st));
    return s.dtype == NSK_BF16 ? d2s_typed<bf16_t>(g, s, ws + p.dx2, dx, accumulate, st)
                               : d2s_typed<float>(g, s, ws + p.dx2, dx, accumulate, st);
}

int stem_wgrad(const ConvGeo &g, const void *x, const void *dy, float *dw, int accumulate, char *ws, hipStream_t st)
{
    const StemGeo s = stem_geo(g);
    const StemPlan p = stem_plan(g, s, NSK_PASS_WGRAD);
    STEM_TRY(space_to_depth(g, s, x, ws + p.x2, st));
    const void *dys = dy;
    if (g.layout == NSK_NCHW) {
        STEM_TRY(launch_nchw_to_nhwc(g.dtype, dy, ws + p.act, g.N, g.K, g.P, g.Q, st));
        dys = ws + p.act;
    }
    WgradArgs a{};
    stem_wgrad_geometry(g, s, &a);
    a.x = ws + p.x2; a.dy = dys; a.part = (float *)(ws + p.part);
    a.rows_per_split = p.rows_per_split;
    a.splits = p.splits;
    if (p.wide)
        STEM_TRY(launch_wgrad_wide(a, st));
    else
        STEM_TRY(launch_wgrad(s.dtype, a, st));
    float *dw2 = (float *)(ws + p.dw2);
    STEM_TRY(launch_wgrad_reduce(a.part, dw2, p.splits, s.K, a.ntaps, SC, (long)a.ntaps * SC, (long)SC, 1L, 0, st));
    long sk, sc, sr, ss;
    filter_strides(g, &sk, &sc, &sr, &ss);
    const int total = s.K * s.C * s.R * s.R;
    hipLaunchKernelGGL(stem_unpack_dw_kernel, dim3((total + 255) / 256), dim3(256), 0, st, dw2, dw, s.K, s.C, s.R, s.pad, s.U,
                       s.umin, sk, sc, sr, ss, accumulate);
    return check_launch();
}

}  // namespace nsk

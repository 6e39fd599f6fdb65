// The C ABI of libnsk: host-side validation, workspace planning and dispatch to the kernels.
// Every check that can be made without touching the device is made before the first HIP call, so
// the error paths behave identically on a machine without a GPU.
#include <limits.h>
#include <stdlib.h>

#include <mutex>

#include "nsk_internal.h"

namespace nsk {

static thread_local int g_last_hip_error = 0;
void set_last_hip_error(hipError_t e) { g_last_hip_error = (int)e; }

namespace {

int out_extent(int in, int pad, int dil, int filt, int stride)
{
    const long span = (long)in + 2L * pad - (long)dil * (filt - 1) - 1;
    return span < 0 ? 0 : (int)(span / stride + 1);
}

// NSK_OK, NSK_ERR_NULL, NSK_ERR_BAD_DESC or NSK_ERR_UNSUPPORTED.  `need_output`: an empty output
// (P or Q = 0) is a bad descriptor for the compute calls, but legal for the extent query.
int conv_geometry(const nsk_conv_desc_t *d, ConvGeo *g, bool need_output)
{
    if (!d) return NSK_ERR_NULL;
    if (d->N < 1 || d->C < 1 || d->H < 1 || d->W < 1 || d->K < 1 || d->R < 1 || d->S < 1) return NSK_ERR_BAD_DESC;
    if (d->stride_h < 1 || d->stride_w < 1 || d->dil_h < 1 || d->dil_w < 1) return NSK_ERR_BAD_DESC;
    if (d->pad_h < 0 || d->pad_w < 0) return NSK_ERR_BAD_DESC;
    if (d->dtype != NSK_F32 && d->dtype != NSK_BF16) return NSK_ERR_BAD_DESC;
    if (d->layout != NSK_NCHW && d->layout != NSK_NHWC) return NSK_ERR_BAD_DESC;
    g->N = d->N; g->C = d->C; g->H = d->H; g->W = d->W; g->K = d->K; g->R = d->R; g->S = d->S;
    g->sh = d->stride_h; g->sw = d->stride_w; g->ph = d->pad_h; g->pw = d->pad_w; g->dh = d->dil_h; g->dw = d->dil_w;
    g->dtype = d->dtype; g->layout = d->layout; g->es = elem_size(d->dtype);
    g->P = out_extent(d->H, d->pad_h, d->dil_h, d->R, d->stride_h);
    g->Q = out_extent(d->W, d->pad_w, d->dil_w, d->S, d->stride_w);
    if (!need_output) return NSK_OK;
    if (g->P < 1 || g->Q < 1) return NSK_ERR_BAD_DESC;
    // Limits of this build: pixel counts index with 32-bit ints, tap tables hold 64 entries with
    // 16-bit offsets, NCHW conversion puts the batch on gridDim.z.
    const long long pix_in = (long long)d->N * d->H * d->W, pix_out = (long long)d->N * g->P * g->Q;
    if (pix_in >= INT_MAX || pix_out >= INT_MAX) return NSK_ERR_UNSUPPORTED;
    if ((long long)d->R * d->S > kMaxTaps) return NSK_ERR_UNSUPPORTED;
    // activations are addressed with 32-bit byte offsets through buffer descriptors
    if (pix_in * d->C * 4 >= 0xFFFFFFFFLL || pix_out * d->K * 4 >= 0xFFFFFFFFLL) return NSK_ERR_UNSUPPORTED;
    if ((long long)(d->R - 1) * d->dil_h > 30000 || (long long)(d->S - 1) * d->dil_w > 30000) return NSK_ERR_UNSUPPORTED;
    if ((long long)d->K * d->R * d->S * d->C >= INT_MAX) return NSK_ERR_UNSUPPORTED;
    if (d->layout == NSK_NCHW && d->N > 65535) return NSK_ERR_UNSUPPORTED;
    g->x_elems = (size_t)pix_in * d->C;
    g->y_elems = (size_t)pix_out * d->K;
    g->w_elems = (size_t)d->K * d->R * d->S * d->C;
    return NSK_OK;
}

// Geometry part of the backward-weight arguments (pointers and split sizes are set by the caller).
void wgrad_geometry(const ConvGeo &g, WgradArgs *a)
{
    a->Nimg = g.N; a->H = g.H; a->W = g.W; a->C = g.C; a->P = g.P; a->Q = g.Q; a->K = g.K;
    a->sh = g.sh; a->sw = g.sw; a->ph = g.ph; a->pw = g.pw;
    a->ntaps = g.R * g.S;
    a->L = g.N * g.P * g.Q;
    for (int r = 0; r < g.R; ++r)
        for (int s = 0; s < g.S; ++s) {
            a->off_h[r * g.S + s] = (short)(r * g.dh);
            a->off_w[r * g.S + s] = (short)(s * g.dw);
        }
}

bool use_wgrad_halo(const ConvGeo &g, const WgradArgs &a)
{
    return wgrad_halo64_applicable(g.dtype, a) && !hooks().no_halo;
}

// Workspace segments (byte offsets, each 256-aligned).
struct ConvPlan {
    size_t act_in = 0;   // NHWC copy of the NCHW input activation (x or dy)
    size_t act_in2 = 0;  // wgrad only: NHWC copy of dy
    size_t filt = 0;     // packed filter
    size_t act_out = 0;  // NHWC result before conversion to NCHW
    size_t part = 0;     // wgrad partial sums
    size_t total = 0;
    int splits = 1, rows_per_split = 0;
    bool halo = false;   // wgrad: the 3x3 64->64 kernel writes one partial per block
    bool wide = false;   // wgrad: the large-tile kernel for wide bf16 layers
    bool stem = false;   // the space-to-depth path plans its own workspace
    size_t act_tmp = 0;  // fused-activation calls on a kernel without the fused load: the applied activation
    bool act_fused = false;
};

// groups > 1: grouped convolution (the filter holds C/groups input channels per output channel and only the generic
// kernels run it).
void fwd_geometry(const ConvGeo &g, IgemmArgs *a);

// act: the call applies a batch-norm + ReLU to x on load (NHWC, one group); where the kernel that takes the layer has no
// fused load the activation is applied into the workspace first.
ConvPlan plan_conv(const ConvGeo &g, int pass, int groups = 1, bool act = false)
{
    ConvPlan p;
    const size_t w_elems = g.w_elems / (size_t)groups;
    p.stem = groups == 1 && stem_applicable(g);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += align_up(bytes);
        return at;
    };
    if (act) {
        // (the pointers only matter for alignment tests: every tensor of these calls is 16-byte aligned)
        if (pass == NSK_PASS_FWD && !p.stem) {
            IgemmArgs a{};
            fwd_geometry(g, &a);
            p.act_fused = igemm_act_fused(g.dtype, a);
        } else if (pass == NSK_PASS_WGRAD && !p.stem) {
            WgradArgs wa{};
            wgrad_geometry(g, &wa);
            p.act_fused = use_wgrad_halo(g, wa) && wgrad_halo64_act_fused(g.dtype, wa);
        }
        if (!p.act_fused) p.act_tmp = take(g.x_elems * g.es);
    }
    if (p.stem) {
        p.total = off + stem_workspace_bytes(g, pass);
        return p;
    }
    const bool nchw = g.layout == NSK_NCHW;
    if (pass == NSK_PASS_FWD) {
        if (nchw) {
            p.act_in = take(g.x_elems * g.es);
            p.filt = take(w_elems * g.es);
            p.act_out = take(g.y_elems * g.es);
        }
    } else if (pass == NSK_PASS_DGRAD) {
        if (nchw) p.act_in = take(g.y_elems * g.es);
        // one packed filter per stride parity class; together they hold every tap once
        p.filt = take(w_elems * g.es + 256 * (size_t)g.sh * g.sw);
        if (nchw) p.act_out = take(g.x_elems * g.es);
    } else {
        if (nchw) {
            p.act_in = take(g.x_elems * g.es);
            p.act_in2 = take(g.y_elems * g.es);
        }
        WgradArgs wa{};
        wgrad_geometry(g, &wa);
        p.halo = groups == 1 && use_wgrad_halo(g, wa);
        p.wide = groups == 1 && !p.halo && wgrad_wide_applicable(g.dtype, wa);
        if (p.halo)
            p.splits = wgrad_halo64_partials(g.dtype, wa, nullptr);
        else if (p.wide)
            p.rows_per_split = wgrad_wide_rows_per_split(wa, &p.splits);
        else
            p.rows_per_split = wgrad_rows_per_split(g.dtype, g.N * g.P * g.Q, g.K, g.R * g.S * (g.C / groups), &p.splits);
        if (groups > 1 && g.C == g.K && (g.C == groups || g.C == 2 * groups || g.C == 4 * groups || g.C == 8 * groups)) {
            // depthwise and its neighbours: the direct kernel runs blocks of 16 channel vectors x one split and wants
            // about four per CU
            const int vec = g.dtype == NSK_BF16 ? 8 : 4, L = g.N * g.P * g.Q;
            const int want = 1024 / ceil_div(ceil_div(g.C, vec), 16) > 0 ? 1024 / ceil_div(ceil_div(g.C, vec), 16) : 1;
            int rows = ceil_div(L, want);
            if (rows < 64) rows = 64;
            p.rows_per_split = ceil_div(rows, 32) * 32;
            p.splits = ceil_div(L, p.rows_per_split);
        }
        // a grouped launch puts groups * splits on gridDim.z
        while ((long)groups * p.splits > 65535) {
            p.rows_per_split *= 2;
            p.splits = ceil_div(g.N * g.P * g.Q, p.rows_per_split);
        }
        p.part = take((size_t)p.splits * w_elems * sizeof(float));
    }
    p.total = off;
    return p;
}

bool misaligned(const void *p) { return ((uintptr_t)p & 15) != 0; }

int check_ws(const void *ws, size_t have, size_t need)
{
    if (need == 0) return NSK_OK;
    if (!ws || have < need) return NSK_ERR_WORKSPACE;
    if (misaligned(ws)) return NSK_ERR_ALIGNMENT;
    return NSK_OK;
}

#define NSK_TRY(expr)                 \
    do {                              \
        const int st__ = (expr);      \
        if (st__ != NSK_OK) return st__; \
    } while (0)

int bn_geometry(const nsk_bn_desc_t *d)
{
    if (!d) return NSK_ERR_NULL;
    if (d->N < 1 || d->C < 1 || d->H < 1 || d->W < 1) return NSK_ERR_BAD_DESC;
    if (d->dtype != NSK_F32 && d->dtype != NSK_BF16) return NSK_ERR_BAD_DESC;
    if (d->layout != NSK_NCHW && d->layout != NSK_NHWC) return NSK_ERR_BAD_DESC;
    if (!(d->eps >= 0.f) || !(d->momentum >= 0.f && d->momentum <= 1.f)) return NSK_ERR_BAD_DESC;
    if (d->relu != 0 && d->relu != 1) return NSK_ERR_BAD_DESC;
    if (d->C > 65535) return NSK_ERR_UNSUPPORTED;
    return NSK_OK;
}

int pool_geometry(const nsk_pool_desc_t *d, int *P, int *Q)
{
    if (!d) return NSK_ERR_NULL;
    if (d->N < 1 || d->C < 1 || d->H < 1 || d->W < 1 || d->R < 1 || d->S < 1) return NSK_ERR_BAD_DESC;
    if (d->stride_h < 1 || d->stride_w < 1 || d->pad_h < 0 || d->pad_w < 0) return NSK_ERR_BAD_DESC;
    if (d->dtype != NSK_F32 && d->dtype != NSK_BF16) return NSK_ERR_BAD_DESC;
    if (d->layout != NSK_NCHW && d->layout != NSK_NHWC) return NSK_ERR_BAD_DESC;
    if ((long)d->R * d->S > 127) return NSK_ERR_UNSUPPORTED;
    *P = out_extent(d->H, d->pad_h, 1, d->R, d->stride_h);
    *Q = out_extent(d->W, d->pad_w, 1, d->S, d->stride_w);
    return NSK_OK;
}

// Geometry part of the forward implicit-GEMM arguments (pointers, byte sizes and statistics are set by the caller).
void fwd_geometry(const ConvGeo &g, IgemmArgs *a)
{
    a->Nimg = g.N; a->Hs = g.H; a->Ws = g.W; a->Cs = g.C;
    a->Mi = g.P; a->Mj = g.Q; a->M = g.N * g.P * g.Q;
    a->mult_h = g.sh; a->add_h = -g.ph; a->mult_w = g.sw; a->add_w = -g.pw;
    a->ntaps = g.R * g.S; a->Ktot = a->ntaps * g.C;
    a->Ngemm = g.K;
    a->Ho = g.P; a->Wo = g.Q; a->Co = g.K; a->osh = 1; a->oa = 0; a->osw = 1; a->ob = 0;
    a->accumulate = 0;
    a->src_bytes = (unsigned)(g.x_elems * g.es);
    a->wpk_bytes = (unsigned)(g.w_elems * g.es);
    for (int r = 0; r < g.R; ++r)
        for (int s = 0; s < g.S; ++s) {
            a->off_h[r * g.S + s] = (short)(r * g.dh);
            a->off_w[r * g.S + s] = (short)(s * g.dw);
        }
}

// The output tensor of a convolution as a batch-norm descriptor of its NHWC form (what the kernels write).
nsk_bn_desc_t output_as_bn(const ConvGeo &g)
{
    nsk_bn_desc_t d{};
    d.N = g.N; d.C = g.K; d.H = g.P; d.W = g.Q;
    d.dtype = g.dtype; d.layout = NSK_NHWC;
    d.eps = 0.f; d.momentum = 0.f; d.relu = 0;
    return d;
}

// Rows of partial sums nsk_conv2d_fwd_stats writes: those of the kernel's own epilogue where it has one (*fused),
// else those of the separate reduction pass over the stored output.
int conv_stats_rows(const ConvGeo &g, bool *fused = nullptr)
{
    int rows = 0;
    if (stem_applicable(g)) {
        rows = stem_stats_rows(g);
    } else {
        IgemmArgs a{};
        fwd_geometry(g, &a);
        rows = igemm_stats_rows(g.dtype, a);
    }
    if (fused) *fused = rows > 0;
    return rows > 0 ? rows : bn_stats_rows(output_as_bn(g));
}

// NSK_OK if C and K split into `groups` equal runs.
int check_groups(const ConvGeo &g, int groups)
{
    if (groups < 1 || g.C % groups != 0 || g.K % groups != 0) return NSK_ERR_BAD_DESC;
    if (groups > 65535) return NSK_ERR_UNSUPPORTED;   // groups ride on gridDim.z
    return NSK_OK;
}

// The input of a fused-activation call as a batch-norm descriptor (for the apply pass of the unfused route).
nsk_bn_desc_t input_as_bn(const ConvGeo &g)
{
    nsk_bn_desc_t d{};
    d.N = g.N; d.C = g.C; d.H = g.H; d.W = g.W;
    d.dtype = g.dtype; d.layout = NSK_NHWC;
    d.eps = 0.f; d.momentum = 0.f; d.relu = 1;
    return d;
}

// NSK_OK if the fused-activation calls take this layer: NHWC, one group, channels the vector kernels handle.
int check_act(const ConvGeo &g, int groups, const float *act)
{
    if (!act) return NSK_OK;
    if (misaligned(act)) return NSK_ERR_ALIGNMENT;
    if (g.layout != NSK_NHWC || groups != 1 || !bn_act_supported(input_as_bn(g))) return NSK_ERR_UNSUPPORTED;
    return NSK_OK;
}

int conv_fwd_impl(const nsk_conv_desc_t *desc, int groups, const void *x, const void *w, void *y, float *stats,
                  void *workspace, size_t workspace_bytes, void *stream, const float *act = nullptr)
{
    ConvGeo g;
    NSK_TRY(conv_geometry(desc, &g, true));
    NSK_TRY(check_groups(g, groups));
    if (!x || !w || !y) return NSK_ERR_NULL;
    if (misaligned(x) || misaligned(w) || misaligned(y)) return NSK_ERR_ALIGNMENT;
    NSK_TRY(check_act(g, groups, act));
    const ConvPlan p = plan_conv(g, NSK_PASS_FWD, groups, act != nullptr);
    const int cg = g.C / groups, kg = g.K / groups;
    NSK_TRY(check_ws(workspace, workspace_bytes, p.total));
    hipStream_t st = (hipStream_t)stream;
    char *ws = (char *)workspace;
    if (act && !p.act_fused) {   // the kernel for this layer has no fused load: apply the activation first
        NSK_TRY(launch_bn_act(input_as_bn(g), x, act, ws + p.act_tmp, st));
        x = ws + p.act_tmp;
        act = nullptr;
        if (p.stem) ws += align_up(g.x_elems * g.es);
    }
    bool fused = false;
    const int rows = stats ? conv_stats_rows(g, &fused) : 0;
    if (p.stem) {
        void *y_nhwc = nullptr;
        NSK_TRY(stem_fwd(g, x, w, y, ws, fused ? stats : nullptr, rows, &y_nhwc, st));
        if (stats && !fused) NSK_TRY(launch_bn_stats(output_as_bn(g), y_nhwc, stats, st));
        return NSK_OK;
    }

    const void *src = x, *filt = w;
    void *dst = y;
    if (g.layout == NSK_NCHW) {
        NSK_TRY(launch_nchw_to_nhwc(g.dtype, x, ws + p.act_in, g.N, g.C, g.H, g.W, st));
        int tap_off[kMaxTaps];
        for (int t = 0; t < g.R * g.S; ++t) tap_off[t] = t;
        NSK_TRY(launch_pack_filter(g.dtype, w, ws + p.filt, g.K, g.R * g.S, cg, (long)cg * g.R * g.S,
                                   (long)g.R * g.S, tap_off, st));
        src = ws + p.act_in;
        filt = ws + p.filt;
        dst = ws + p.act_out;
    }
    IgemmArgs a{};
    fwd_geometry(g, &a);
    a.src = src; a.wpk = filt; a.out = dst;
    if (groups > 1) {   // `groups` problems of cg -> kg channels on channel runs of the same tensors
        a.groups = groups;
        a.src_ld = g.C;
        a.Cs = cg;
        a.Ktot = a.ntaps * cg;
        a.Ngemm = kg;
        a.wpk_bytes = (unsigned)(g.w_elems / (size_t)groups * g.es);
    }
    if (fused) {
        a.stats = stats;
        a.stats_rows = rows;
    }
    a.act = act;
    NSK_TRY(launch_igemm(g.dtype, a, st));
    if (stats && !fused) NSK_TRY(launch_bn_stats(output_as_bn(g), dst, stats, st));
    if (g.layout == NSK_NCHW) NSK_TRY(launch_nhwc_to_nchw(g.dtype, dst, y, g.N, g.K, g.P, g.Q, 0, st));
    return NSK_OK;
}

}  // namespace
}  // namespace nsk

using namespace nsk;

namespace nsk {
namespace {
TestHooks g_hooks;
bool g_hooks_read = false;

void read_hooks()
{
    auto on = [](const char *name) { return getenv(name) != nullptr; };
    auto num = [](const char *name) { const char *e = getenv(name); return e ? atoll(e) : -1LL; };
    TestHooks h{};
    h.no_big = on("NSK_NO_BIG");
    h.no_big_multi = on("NSK_NO_BIG_MULTI");
    h.no_pw = on("NSK_NO_PW");
    h.no_halo = on("NSK_NO_HALO");
    h.no_fs = on("NSK_NO_FS");
    h.no_halo_wide = on("NSK_NO_HALO_WIDE");
    h.halo_wide_always = on("NSK_HALO_WIDE_ALWAYS");
    h.halo_single = on("NSK_HALO_SINGLE");
    h.no_stem = on("NSK_NO_STEM");
    h.no_stem_halo = on("NSK_NO_STEM_HALO");
    h.no_tiny = on("NSK_NO_TINY");
    h.no_wide = on("NSK_NO_WIDE");
    h.no_depthwise = on("NSK_NO_DEPTHWISE");
    h.depthwise_no_rows = on("NSK_DEPTHWISE_NO_ROWS");
    h.depthwise_no_cols = on("NSK_DEPTHWISE_NO_COLS");
    h.pool_general = on("NSK_POOL_GENERAL");
    h.stats_always = on("NSK_STATS_ALWAYS");
    h.reduce4 = on("NSK_REDUCE4");
    h.wh_no_split = on("NSK_WH_NO_SPLIT");
    h.big_min_tiles = num("NSK_BIG_MIN_TILES");
    h.pw_min_rows = num("NSK_PW_MIN_ROWS");
    h.wide_min_rows = num("NSK_WIDE_MIN_ROWS");
    const long long tile = num("NSK_IGEMM_TILE");
    h.igemm_tile = tile > 0 ? (int)tile : 0;
    g_hooks = h;
    g_hooks_read = true;
}
}  // namespace

const TestHooks &hooks()
{
    if (!g_hooks_read) read_hooks();
    return g_hooks;
}
}  // namespace nsk

extern "C" {

int nsk_version(void) { return 100; }

void nsk_test_hooks_reload(void) { nsk::read_hooks(); }

const char *nsk_status_string(int status)
{
    switch (status) {
    case NSK_OK: return "ok";
    case NSK_ERR_NULL: return "a required pointer is NULL";
    case NSK_ERR_BAD_DESC: return "descriptor field out of range or empty output";
    case NSK_ERR_UNSUPPORTED: return "valid request not supported by this build";
    case NSK_ERR_WORKSPACE: return "workspace missing or too small";
    case NSK_ERR_ALIGNMENT: return "pointer not 16-byte aligned";
    case NSK_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

int nsk_last_hip_error(void) { return g_last_hip_error; }

int nsk_conv2d_out_dims(const nsk_conv_desc_t *desc, int *P, int *Q)
{
    if (!desc || !P || !Q) return NSK_ERR_NULL;
    ConvGeo g;
    NSK_TRY(conv_geometry(desc, &g, false));
    *P = g.P;
    *Q = g.Q;
    return NSK_OK;
}

size_t nsk_conv2d_workspace_bytes(const nsk_conv_desc_t *desc, int pass)
{
    ConvGeo g;
    if (pass < NSK_PASS_FWD || pass > NSK_PASS_WGRAD) return 0;
    if (conv_geometry(desc, &g, true) != NSK_OK) return 0;
    return plan_conv(g, pass).total;
}

int nsk_conv2d_fwd(const nsk_conv_desc_t *desc, const void *x, const void *w, void *y, void *workspace,
                   size_t workspace_bytes, void *stream)
{
    return conv_fwd_impl(desc, 1, x, w, y, nullptr, workspace, workspace_bytes, stream);
}

int nsk_conv2d_stats_rows(const nsk_conv_desc_t *desc)
{
    ConvGeo g;
    if (conv_geometry(desc, &g, true) != NSK_OK) return 0;
    return conv_stats_rows(g);
}

int nsk_conv2d_fwd_stats(const nsk_conv_desc_t *desc, const void *x, const void *w, void *y, float *stats,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    if (!stats) return NSK_ERR_NULL;
    if (misaligned(stats)) return NSK_ERR_ALIGNMENT;
    return conv_fwd_impl(desc, 1, x, w, y, stats, workspace, workspace_bytes, stream);
}

static int conv_dgrad_impl(const nsk_conv_desc_t *desc, int groups, const void *dy, const void *w, void *dx,
                           int accumulate, void *workspace, size_t workspace_bytes, void *stream)
{
    ConvGeo g;
    NSK_TRY(conv_geometry(desc, &g, true));
    NSK_TRY(check_groups(g, groups));
    if (!dy || !w || !dx) return NSK_ERR_NULL;
    if (accumulate != 0 && accumulate != 1) return NSK_ERR_BAD_DESC;
    if (misaligned(dy) || misaligned(w) || misaligned(dx)) return NSK_ERR_ALIGNMENT;
    const ConvPlan p = plan_conv(g, NSK_PASS_DGRAD, groups);
    const int cg = g.C / groups, kg = g.K / groups;   // channels of one group (all of them for a plain convolution)
    NSK_TRY(check_ws(workspace, workspace_bytes, p.total));
    hipStream_t st = (hipStream_t)stream;
    char *ws = (char *)workspace;
    const bool nchw = g.layout == NSK_NCHW;
    if (p.stem) return stem_dgrad(g, dy, w, dx, accumulate, ws, st);

    const void *src = dy;
    void *dst = dx;
    int acc_kernel = accumulate;
    if (nchw) {
        NSK_TRY(launch_nchw_to_nhwc(g.dtype, dy, ws + p.act_in, g.N, g.K, g.P, g.Q, st));
        src = ws + p.act_in;
        dst = ws + p.act_out;
        acc_kernel = 0;  // the conversion back to NCHW does the add
    }
    // dx[h] with h = a + sh*i receives dy[p] * w[r] exactly for the taps r with
    // (a + ph - r*dh) divisible by sh, at p = i + (a + ph - r*dh)/sh: one dense sub-problem per
    // residue class (a, b) of (h mod sh, w mod sw), so no multiply is spent on inserted zeros.
    // Geometry of one class (everything but the pointers); returns its number of taps.
    auto class_args = [&](int ca, int cb, IgemmArgs *a, int *tap_off) {
        int nt = 0;
        for (int r = 0; r < g.R; ++r) {
            const int th = ca + g.ph - r * g.dh;
            if (((th % g.sh) + g.sh) % g.sh != 0) continue;
            for (int s = 0; s < g.S; ++s) {
                const int tw = cb + g.pw - s * g.dw;
                if (((tw % g.sw) + g.sw) % g.sw != 0) continue;
                a->off_h[nt] = (short)(th / g.sh);  // exact division, may be negative
                a->off_w[nt] = (short)(tw / g.sw);
                tap_off[nt] = nchw ? r * g.S + s : (r * g.S + s) * cg;
                ++nt;
            }
        }
        a->Nimg = g.N; a->Hs = g.P; a->Ws = g.Q; a->Cs = kg;
        a->Mi = ca < g.H ? (g.H - ca + g.sh - 1) / g.sh : 0;
        a->Mj = cb < g.W ? (g.W - cb + g.sw - 1) / g.sw : 0;
        a->M = g.N * a->Mi * a->Mj;
        a->mult_h = 1; a->add_h = 0; a->mult_w = 1; a->add_w = 0;
        a->ntaps = nt; a->Ktot = nt * kg;
        a->Ngemm = cg;
        if (groups > 1) {
            a->groups = groups;
            a->src_ld = g.K;
        }
        a->Ho = g.H; a->Wo = g.W; a->Co = g.C; a->osh = g.sh; a->oa = ca; a->osw = g.sw; a->ob = cb;
        a->accumulate = acc_kernel;
        a->src_bytes = (unsigned)(g.y_elems * g.es);
        a->wpk_bytes = (unsigned)((size_t)g.C * nt * kg * g.es);
        return nt;
    };
    // Stride 2 with every tap in class (0, 0) (a 1x1 layer): the other three classes are plain zeros, which the
    // short-reduction kernel writes along with class (0, 0) when it takes that class.
    bool zero_cell = false;
    if (g.sh == 2 && g.sw == 2 && !acc_kernel && groups == 1) {
        IgemmArgs a{};
        int tap_off[kMaxTaps];
        bool others_empty = true;
        for (int c = 1; c < 4; ++c) others_empty = others_empty && class_args(c >> 1, c & 1, &a, tap_off) == 0;
        if (others_empty && class_args(0, 0, &a, tap_off) > 0) {
            a.src = src; a.wpk = ws + p.filt; a.out = dst;
            zero_cell = conv_pw_applicable(g.dtype, a);
        }
    }
    // element (k, tap, c) of the filter: k * w_sc + tap_off + c * w_sn; one group's filters are w_gstep elements long
    const long w_sn = nchw ? (long)g.R * g.S : 1L, w_sc = (long)g.R * g.S * cg;
    const long w_gstep = (long)kg * w_sc;
    size_t filt_off = p.filt;
    // classes with taps: filters are packed first, then the launches follow (one for all classes where the large-tile
    // kernel takes them together)
    IgemmArgs pending[4];
    int n_pending = 0;
    const bool may_merge = g.sh * g.sw <= 4;
    int pk_taps[4][kMaxTaps], pk_nt[4];
    void *pk_out[4];
    for (int ca = 0; ca < g.sh; ++ca)
        for (int cb = 0; cb < g.sw; ++cb) {
            IgemmArgs a{};
            int tap_off[kMaxTaps];
            const int nt = class_args(ca, cb, &a, tap_off);
            if (a.Mi == 0 || a.Mj == 0) continue;
            if (nt == 0 && accumulate && !nchw) continue;  // nothing to add
            if (nt == 0) {   // no tap reaches this class: plain zero fill
                if (!zero_cell)
                    NSK_TRY(launch_zero_class(g.dtype, dst, g.N, g.H, g.W, g.C, a.Mi, a.Mj, g.sh, ca, g.sw, cb, st));
                continue;
            }
            // packed filter of this class: [c][tap][k] with element (c, t, k) = w[c*sn + tap_off[t] + k*sc]
            a.src = src; a.wpk = ws + filt_off; a.out = dst;
            a.zero_cell = zero_cell ? 1 : 0;
            if (may_merge) {
                for (int t = 0; t < kMaxTaps; ++t) pk_taps[n_pending][t] = t < nt ? tap_off[t] : 0;
                pk_nt[n_pending] = nt;
                pk_out[n_pending] = ws + filt_off;
                pending[n_pending++] = a;
            } else {
                int taps1[1][kMaxTaps];
                for (int t = 0; t < kMaxTaps; ++t) taps1[0][t] = t < nt ? tap_off[t] : 0;
                void *out1[1] = {ws + filt_off};
                NSK_TRY(launch_pack_filters_grouped(g.dtype, 1, w, out1, cg, &nt, kg, w_sn, w_sc, taps1, groups, w_gstep, st));
                NSK_TRY(launch_igemm(g.dtype, a, st));
            }
            filt_off += align_up((size_t)g.C * nt * kg * g.es);
        }
    // one packing launch for all classes, then their multiplies
    if (n_pending > 0)
        NSK_TRY(launch_pack_filters_grouped(g.dtype, n_pending, w, pk_out, cg, pk_nt, kg, w_sn, w_sc, pk_taps, groups, w_gstep, st));
    if (n_pending == 4 && groups == 1 && fs64_dgrad_s2_applicable(g.dtype, pending, n_pending)) {
        NSK_TRY(launch_fs64_dgrad_s2(pending, n_pending, st));
    } else if (n_pending > 1 && groups == 1 && halo_wide_multi_applicable(g.dtype, pending, n_pending)) {
        NSK_TRY(launch_halo_wide_multi(pending, n_pending, st));
    } else if (n_pending > 1 && groups == 1 && igemm_big_multi_applicable(g.dtype, pending, n_pending)) {
        NSK_TRY(launch_igemm_big_multi(pending, n_pending, st));
    } else {
        for (int i = 0; i < n_pending; ++i) NSK_TRY(launch_igemm(g.dtype, pending[i], st));
    }
    if (nchw) NSK_TRY(launch_nhwc_to_nchw(g.dtype, dst, dx, g.N, g.C, g.H, g.W, accumulate, st));
    return NSK_OK;
}

static int conv_wgrad_impl(const nsk_conv_desc_t *desc, int groups, const void *x, const void *dy, float *dw,
                           int accumulate, void *workspace, size_t workspace_bytes, void *stream,
                           const float *act = nullptr)
{
    ConvGeo g;
    NSK_TRY(conv_geometry(desc, &g, true));
    NSK_TRY(check_groups(g, groups));
    if (!x || !dy || !dw) return NSK_ERR_NULL;
    if (accumulate != 0 && accumulate != 1) return NSK_ERR_BAD_DESC;
    if (misaligned(x) || misaligned(dy) || misaligned(dw)) return NSK_ERR_ALIGNMENT;
    NSK_TRY(check_act(g, groups, act));
    const ConvPlan p = plan_conv(g, NSK_PASS_WGRAD, groups, act != nullptr);
    const int cg = g.C / groups, kg = g.K / groups;
    NSK_TRY(check_ws(workspace, workspace_bytes, p.total));
    hipStream_t st = (hipStream_t)stream;
    char *ws = (char *)workspace;
    if (act && !p.act_fused) {   // the kernel for this layer has no fused load: apply the activation first
        NSK_TRY(launch_bn_act(input_as_bn(g), x, act, ws + p.act_tmp, st));
        x = ws + p.act_tmp;
        act = nullptr;
        if (p.stem) ws += align_up(g.x_elems * g.es);
    }
    const bool nchw = g.layout == NSK_NCHW;
    if (p.stem) return stem_wgrad(g, x, dy, dw, accumulate, ws, st);
    const void *xs = x, *dys = dy;
    if (nchw) {
        NSK_TRY(launch_nchw_to_nhwc(g.dtype, x, ws + p.act_in, g.N, g.C, g.H, g.W, st));
        NSK_TRY(launch_nchw_to_nhwc(g.dtype, dy, ws + p.act_in2, g.N, g.K, g.P, g.Q, st));
        xs = ws + p.act_in;
        dys = ws + p.act_in2;
    }
    WgradArgs a{};
    a.x = xs; a.dy = dys; a.part = (float *)(ws + p.part);
    a.act = act;
    wgrad_geometry(g, &a);
    a.rows_per_split = p.rows_per_split;
    a.splits = p.splits;
    if (groups > 1) {   // `groups` problems of cg x kg channels; their partial sums stack to [splits][K][taps * cg]
        a.groups = groups;
        a.ldx = g.C;
        a.ldy = g.K;
        a.C = cg;
        a.K = kg;
    }
    if (p.halo)
        NSK_TRY(launch_wgrad_halo64(g.dtype, a, st));
    else if (p.wide)
        NSK_TRY(launch_wgrad_wide(a, st));
    else
        NSK_TRY(launch_wgrad(g.dtype, a, st));
    const long RS = (long)g.R * g.S;
    if (nchw)
        NSK_TRY(launch_wgrad_reduce(a.part, dw, p.splits, g.K, a.ntaps, cg, (long)cg * RS, 1L, RS, accumulate, st));
    else
        NSK_TRY(launch_wgrad_reduce(a.part, dw, p.splits, g.K, a.ntaps, cg, RS * cg, (long)cg, 1L, accumulate, st));
    return NSK_OK;
}

int nsk_conv2d_dgrad(const nsk_conv_desc_t *desc, const void *dy, const void *w, void *dx, int accumulate,
                     void *workspace, size_t workspace_bytes, void *stream)
{
    return conv_dgrad_impl(desc, 1, dy, w, dx, accumulate, workspace, workspace_bytes, stream);
}

int nsk_conv2d_wgrad(const nsk_conv_desc_t *desc, const void *x, const void *dy, float *dw, int accumulate,
                     void *workspace, size_t workspace_bytes, void *stream)
{
    return conv_wgrad_impl(desc, 1, x, dy, dw, accumulate, workspace, workspace_bytes, stream);
}

int nsk_conv2d_wgrad_act(const nsk_conv_desc_t *desc, const void *x, const float *coeffs, const void *dy, float *dw,
                         int accumulate, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!coeffs) return NSK_ERR_NULL;
    return conv_wgrad_impl(desc, 1, x, dy, dw, accumulate, workspace, workspace_bytes, stream, coeffs);
}

size_t nsk_conv2d_grouped_workspace_bytes(const nsk_conv_desc_t *desc, int groups, int pass)
{
    ConvGeo g;
    if (pass < NSK_PASS_FWD || pass > NSK_PASS_WGRAD) return 0;
    if (conv_geometry(desc, &g, true) != NSK_OK || check_groups(g, groups) != NSK_OK) return 0;
    return plan_conv(g, pass, groups).total;
}

int nsk_conv2d_grouped_fwd(const nsk_conv_desc_t *desc, int groups, const void *x, const void *w, void *y,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    return conv_fwd_impl(desc, groups, x, w, y, nullptr, workspace, workspace_bytes, stream);
}

int nsk_conv2d_grouped_dgrad(const nsk_conv_desc_t *desc, int groups, const void *dy, const void *w, void *dx,
                             int accumulate, void *workspace, size_t workspace_bytes, void *stream)
{
    return conv_dgrad_impl(desc, groups, dy, w, dx, accumulate, workspace, workspace_bytes, stream);
}

int nsk_conv2d_grouped_wgrad(const nsk_conv_desc_t *desc, int groups, const void *x, const void *dy, float *dw,
                             int accumulate, void *workspace, size_t workspace_bytes, void *stream)
{
    return conv_wgrad_impl(desc, groups, x, dy, dw, accumulate, workspace, workspace_bytes, stream);
}

size_t nsk_bn_workspace_bytes(const nsk_bn_desc_t *desc, int pass)
{
    if (pass != NSK_BN_FWD && pass != NSK_BN_BWD) return 0;
    if (bn_geometry(desc) != NSK_OK) return 0;
    const size_t G = (size_t)bn_partial_blocks(*desc);
    const size_t floats = align_up((2 * G * desc->C + 4 * (size_t)desc->C) * sizeof(float));
    return floats + (pass == NSK_BN_BWD ? align_up(bn_mask_bytes(*desc)) : 0);
}

int nsk_bn_relu_add_fwd(const nsk_bn_desc_t *desc, const void *x, const void *residual, const float *gamma,
                        const float *beta, void *out, float *save_mean, float *save_invstd, float *running_mean,
                        float *running_var, void *workspace, size_t workspace_bytes, void *stream)
{
    NSK_TRY(bn_geometry(desc));
    if (!x || !gamma || !beta || !out || !save_mean || !save_invstd) return NSK_ERR_NULL;
    if ((running_mean == nullptr) != (running_var == nullptr)) return NSK_ERR_NULL;
    if (misaligned(x) || misaligned(residual) || misaligned(out) || misaligned(gamma) || misaligned(beta) ||
        misaligned(save_mean) || misaligned(save_invstd) || misaligned(running_mean) || misaligned(running_var))
        return NSK_ERR_ALIGNMENT;
    NSK_TRY(check_ws(workspace, workspace_bytes, nsk_bn_workspace_bytes(desc, NSK_BN_FWD)));
    return launch_bn_fwd(*desc, x, residual, gamma, beta, out, save_mean, save_invstd, running_mean, running_var,
                         workspace, nullptr, nullptr, 0, (hipStream_t)stream);
}

// ---- nsk_bn_relu_add_fwd for callers that cannot allocate: the partial sums live in a file-scope device array.
// The array's name is a host-side stand-in, not a device address: host code only ever uses the address that
// hipGetSymbolAddress returns for the current device (each GPU holds its own copy at its own address).
#define NSK_STATIC_SCRATCH_BYTES (8u << 20)
static __device__ __align__(256) unsigned char scratch[NSK_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device, looked up once per device.
int static_scratch(void **ptr)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        nsk::set_last_hip_error(e);
        return NSK_ERR_HIP;
    }
    if (dev < 0 || dev >= kMaxDevices) return NSK_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (g_scratch_ptr[dev] == nullptr) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || p == nullptr) {
            nsk::set_last_hip_error(e);
            return NSK_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return NSK_OK;
}
}  // namespace

size_t nsk_static_scratch_bytes(void) { return NSK_STATIC_SCRATCH_BYTES; }

int nsk_bn_relu_add_fwd_static(const nsk_bn_desc_t *desc, const void *x, const void *residual, const float *gamma,
                               const float *beta, void *out, float *save_mean, float *save_invstd,
                               float *running_mean, float *running_var, void *stream)
{
    NSK_TRY(bn_geometry(desc));
    if (!x || !gamma || !beta || !out || !save_mean || !save_invstd) return NSK_ERR_NULL;
    if ((running_mean == nullptr) != (running_var == nullptr)) return NSK_ERR_NULL;
    if (misaligned(x) || misaligned(residual) || misaligned(out) || misaligned(gamma) || misaligned(beta) ||
        misaligned(save_mean) || misaligned(save_invstd) || misaligned(running_mean) || misaligned(running_var))
        return NSK_ERR_ALIGNMENT;
    // the partial sums of this descriptor must fit the static array (checked before any HIP call)
    if (nsk_bn_workspace_bytes(desc, NSK_BN_FWD) > NSK_STATIC_SCRATCH_BYTES) return NSK_ERR_WORKSPACE;
    void *ws = nullptr;
    NSK_TRY(static_scratch(&ws));
    // every partial sum the finalize kernel reads is written by the reduction of the same call: nothing to clear
    return launch_bn_fwd(*desc, x, residual, gamma, beta, out, save_mean, save_invstd, running_mean, running_var, ws,
                         nullptr, nullptr, 0, (hipStream_t)stream);
}

// ---- batch-norm + ReLU applied by the CONSUMERS of a convolution's raw output (the normalised activation is never stored)
int nsk_bn_fwd_coeffs(const nsk_bn_desc_t *desc, const float *gamma, const float *beta, const float *stats,
                      int stats_rows, float *save_mean, float *save_invstd, float *running_mean, float *running_var,
                      float *coeffs, void *workspace, size_t workspace_bytes, void *stream)
{
    NSK_TRY(bn_geometry(desc));
    if (!gamma || !beta || !stats || !save_mean || !save_invstd || !coeffs) return NSK_ERR_NULL;
    if (stats_rows < 1) return NSK_ERR_BAD_DESC;
    if ((running_mean == nullptr) != (running_var == nullptr)) return NSK_ERR_NULL;
    if (misaligned(gamma) || misaligned(beta) || misaligned(stats) || misaligned(save_mean) || misaligned(save_invstd) ||
        misaligned(running_mean) || misaligned(running_var) || misaligned(coeffs))
        return NSK_ERR_ALIGNMENT;
    NSK_TRY(check_ws(workspace, workspace_bytes, nsk_bn_workspace_bytes(desc, NSK_BN_FWD)));
    return launch_bn_coeffs(*desc, gamma, beta, stats, stats_rows, save_mean, save_invstd, running_mean, running_var,
                            coeffs, workspace, (hipStream_t)stream);
}

int nsk_conv2d_act_supported(const nsk_conv_desc_t *desc)
{
    ConvGeo g;
    if (conv_geometry(desc, &g, true) != NSK_OK) return 0;
    return g.layout == NSK_NHWC && bn_act_supported(input_as_bn(g)) ? 1 : 0;
}

size_t nsk_conv2d_act_workspace_bytes(const nsk_conv_desc_t *desc, int pass)
{
    ConvGeo g;
    if (pass != NSK_PASS_FWD && pass != NSK_PASS_WGRAD) return 0;
    if (conv_geometry(desc, &g, true) != NSK_OK) return 0;
    if (g.layout != NSK_NHWC || !bn_act_supported(input_as_bn(g))) return 0;
    return plan_conv(g, pass, 1, true).total;
}

int nsk_conv2d_fwd_act(const nsk_conv_desc_t *desc, const void *x, const float *coeffs, const void *w, void *y,
                       float *stats, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!coeffs) return NSK_ERR_NULL;
    if (misaligned(stats)) return NSK_ERR_ALIGNMENT;
    return conv_fwd_impl(desc, 1, x, w, y, stats, workspace, workspace_bytes, stream, coeffs);
}

int nsk_bn_relu_bwd_act(const nsk_bn_desc_t *desc, const void *x, const float *coeffs, const void *dout,
                        const float *gamma, const float *save_mean, const float *save_invstd, void *dx, float *dgamma,
                        float *dbeta, void *workspace, size_t workspace_bytes, void *stream)
{
    NSK_TRY(bn_geometry(desc));
    if (!x || !coeffs || !dout || !gamma || !save_mean || !save_invstd || !dx || !dgamma || !dbeta) return NSK_ERR_NULL;
    if (misaligned(x) || misaligned(coeffs) || misaligned(dout) || misaligned(dx) || misaligned(gamma) ||
        misaligned(save_mean) || misaligned(save_invstd) || misaligned(dgamma) || misaligned(dbeta))
        return NSK_ERR_ALIGNMENT;
    if (!desc->relu || desc->layout != NSK_NHWC || !bn_act_supported(*desc)) return NSK_ERR_UNSUPPORTED;
    NSK_TRY(check_ws(workspace, workspace_bytes, nsk_bn_workspace_bytes(desc, NSK_BN_BWD)));
    return launch_bn_bwd(*desc, x, nullptr, dout, gamma, save_mean, save_invstd, dx, nullptr, dgamma, dbeta, workspace,
                         nullptr, (hipStream_t)stream, coeffs);
}

int nsk_bn_relu_add_bwd(const nsk_bn_desc_t *desc, const void *x, const void *out, const void *dout,
                        const float *gamma, const float *save_mean, const float *save_invstd, void *dx,
                        void *dresidual, float *dgamma, float *dbeta, void *workspace, size_t workspace_bytes,
                        void *stream)
{
    NSK_TRY(bn_geometry(desc));
    if (!x || !dout || !gamma || !save_mean || !save_invstd || !dx || !dgamma || !dbeta) return NSK_ERR_NULL;
    if (desc->relu && !out) return NSK_ERR_NULL;
    if (misaligned(x) || misaligned(out) || misaligned(dout) || misaligned(dx) || misaligned(dresidual) ||
        misaligned(gamma) || misaligned(save_mean) || misaligned(save_invstd) || misaligned(dgamma) ||
        misaligned(dbeta))
        return NSK_ERR_ALIGNMENT;
    NSK_TRY(check_ws(workspace, workspace_bytes, nsk_bn_workspace_bytes(desc, NSK_BN_BWD)));
    return launch_bn_bwd(*desc, x, out, dout, gamma, save_mean, save_invstd, dx, dresidual, dgamma, dbeta, workspace,
                         nullptr, (hipStream_t)stream);
}

size_t nsk_bn_mask_bytes(const nsk_bn_desc_t *desc)
{
    if (bn_geometry(desc) != NSK_OK) return 0;
    return bn_mask_bytes(*desc);
}

int nsk_bn_relu_add_fwd_mask(const nsk_bn_desc_t *desc, const void *x, const void *residual, const float *gamma,
                             const float *beta, void *out, unsigned char *relu_mask, float *save_mean,
                             float *save_invstd, float *running_mean, float *running_var, void *workspace,
                             size_t workspace_bytes, void *stream)
{
    NSK_TRY(bn_geometry(desc));
    if (bn_mask_bytes(*desc) == 0) return NSK_ERR_UNSUPPORTED;
    if (!x || !gamma || !beta || !out || !relu_mask || !save_mean || !save_invstd) return NSK_ERR_NULL;
    if ((running_mean == nullptr) != (running_var == nullptr)) return NSK_ERR_NULL;
    if (misaligned(x) || misaligned(residual) || misaligned(out) || misaligned(relu_mask) || misaligned(gamma) ||
        misaligned(beta) || misaligned(save_mean) || misaligned(save_invstd) || misaligned(running_mean) ||
        misaligned(running_var))
        return NSK_ERR_ALIGNMENT;
    NSK_TRY(check_ws(workspace, workspace_bytes, nsk_bn_workspace_bytes(desc, NSK_BN_FWD)));
    return launch_bn_fwd(*desc, x, residual, gamma, beta, out, save_mean, save_invstd, running_mean, running_var,
                         workspace, relu_mask, nullptr, 0, (hipStream_t)stream);
}

int nsk_bn_relu_add_fwd_stats(const nsk_bn_desc_t *desc, const void *x, const void *residual, const float *gamma,
                              const float *beta, void *out, unsigned char *relu_mask, float *save_mean,
                              float *save_invstd, float *running_mean, float *running_var, const float *stats,
                              int stats_rows, void *workspace, size_t workspace_bytes, void *stream)
{
    NSK_TRY(bn_geometry(desc));
    if (!x || !gamma || !beta || !out || !save_mean || !save_invstd || !stats) return NSK_ERR_NULL;
    if (stats_rows < 1) return NSK_ERR_BAD_DESC;
    if (relu_mask && bn_mask_bytes(*desc) == 0) return NSK_ERR_UNSUPPORTED;
    if ((running_mean == nullptr) != (running_var == nullptr)) return NSK_ERR_NULL;
    if (misaligned(x) || misaligned(residual) || misaligned(out) || misaligned(relu_mask) || misaligned(gamma) ||
        misaligned(beta) || misaligned(save_mean) || misaligned(save_invstd) || misaligned(running_mean) ||
        misaligned(running_var) || misaligned(stats))
        return NSK_ERR_ALIGNMENT;
    NSK_TRY(check_ws(workspace, workspace_bytes, nsk_bn_workspace_bytes(desc, NSK_BN_FWD)));
    return launch_bn_fwd(*desc, x, residual, gamma, beta, out, save_mean, save_invstd, running_mean, running_var,
                         workspace, relu_mask, stats, stats_rows, (hipStream_t)stream);
}

int nsk_bn_relu_add_bwd_mask(const nsk_bn_desc_t *desc, const void *x, const unsigned char *relu_mask, const void *dout,
                             const float *gamma, const float *save_mean, const float *save_invstd, void *dx,
                             void *dresidual, float *dgamma, float *dbeta, void *workspace, size_t workspace_bytes,
                             void *stream)
{
    NSK_TRY(bn_geometry(desc));
    if (bn_mask_bytes(*desc) == 0) return NSK_ERR_UNSUPPORTED;
    if (!x || !relu_mask || !dout || !gamma || !save_mean || !save_invstd || !dx || !dgamma || !dbeta) return NSK_ERR_NULL;
    if (misaligned(x) || misaligned(relu_mask) || misaligned(dout) || misaligned(dx) || misaligned(dresidual) ||
        misaligned(gamma) || misaligned(save_mean) || misaligned(save_invstd) || misaligned(dgamma) || misaligned(dbeta))
        return NSK_ERR_ALIGNMENT;
    NSK_TRY(check_ws(workspace, workspace_bytes, nsk_bn_workspace_bytes(desc, NSK_BN_BWD)));
    return launch_bn_bwd(*desc, x, nullptr, dout, gamma, save_mean, save_invstd, dx, dresidual, dgamma, dbeta, workspace,
                         relu_mask, (hipStream_t)stream);
}

int nsk_maxpool2d_out_dims(const nsk_pool_desc_t *desc, int *P, int *Q)
{
    if (!desc || !P || !Q) return NSK_ERR_NULL;
    int p, q;
    NSK_TRY(pool_geometry(desc, &p, &q));
    *P = p;
    *Q = q;
    return NSK_OK;
}

int nsk_maxpool2d_fwd(const nsk_pool_desc_t *desc, const void *x, void *y, signed char *idx, void *stream)
{
    int P, Q;
    NSK_TRY(pool_geometry(desc, &P, &Q));
    if (P < 1 || Q < 1) return NSK_ERR_BAD_DESC;
    if (!x || !y || !idx) return NSK_ERR_NULL;
    if (misaligned(x) || misaligned(y) || misaligned(idx)) return NSK_ERR_ALIGNMENT;
    return launch_maxpool_fwd(*desc, P, Q, x, y, idx, (hipStream_t)stream);
}

int nsk_maxpool2d_bwd(const nsk_pool_desc_t *desc, const void *dy, const signed char *idx, void *dx, void *stream)
{
    int P, Q;
    NSK_TRY(pool_geometry(desc, &P, &Q));
    if (P < 1 || Q < 1) return NSK_ERR_BAD_DESC;
    if (!dy || !idx || !dx) return NSK_ERR_NULL;
    if (misaligned(dy) || misaligned(idx) || misaligned(dx)) return NSK_ERR_ALIGNMENT;
    return launch_maxpool_bwd(*desc, P, Q, dy, idx, dx, (hipStream_t)stream);
}

}  // extern "C"

// Internal declarations shared by the translation units of libnsk (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <type_traits>

#include "nsk.h"

namespace nsk {

typedef __bf16 bf16_t;
typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kMaxTaps = 64;    // R*S of one launch (a 7x7 filter has 49)
constexpr int kMaxBnChannels = 4096;

inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline size_t elem_size(int dtype) { return dtype == NSK_BF16 ? 2 : 4; }

// Compile-time loop: f(std::integral_constant<int, B>), ..., f(std::integral_constant<int, E - 1>).  For loop bodies
// whose index must be a constant expression (register arrays, per-iteration schedules chosen with `if constexpr`).
template <int B, int E, typename F> __device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

// Block-wide barrier that orders LDS traffic only.  __syncthreads() also drains the wavefront's global loads
// (its fence covers global memory), which would end every register prefetch at each barrier; kernels whose
// wavefronts exchange data through LDS alone use this one and keep their loads in flight across it.
__device__ inline void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Test and A/B switches: environment variables NSK_*, read ONCE (first use, or nsk_test_hooks_reload()) and never on
// the launch path.  Each one only narrows or widens the choice among kernels that all compute the same result.
struct TestHooks {
    bool no_big, no_big_multi, no_pw, no_halo, no_fs, no_halo_wide, halo_wide_always, halo_single, no_stem, no_stem_halo,
        no_tiny, no_wide, no_depthwise, depthwise_no_rows, depthwise_no_cols, pool_general, stats_always, reduce4,
        wh_no_split;
    long long big_min_tiles, pw_min_rows, wide_min_rows;   // -1: not set
    int igemm_tile;                                         // 0: not set
};
const TestHooks &hooks();

void set_last_hip_error(hipError_t e);
// Returns NSK_OK or records the error and returns NSK_ERR_HIP.
inline int check_launch()
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_last_hip_error(e);
        return NSK_ERR_HIP;
    }
    return NSK_OK;
}

// Validated geometry of one convolution descriptor.
struct ConvGeo {
    int N, C, H, W, K, R, S, sh, sw, ph, pw, dh, dw, P, Q;
    int dtype, layout;
    size_t es;
    size_t x_elems, y_elems, w_elems;
};

// ------------------------------------------------------------------ implicit GEMM (fwd, dgrad)
// One launch computes, for every GEMM row m = (img, i, j) with i < Mi, j < Mj and every
// column n < Ngemm:
//   acc[m][n] = sum over taps t and channels c of
//               src[img][i*mult_h + add_h + off_h[t]][j*mult_w + add_w + off_w[t]][c] * wpk[n][t][c]
// (source positions outside [0,Hs) x [0,Ws) count as zero) and stores it, converted to the
// element type, at out[img][i*osh + oa][j*osw + ob][n], adding the old value if `accumulate`.
struct IgemmArgs {
    const void *src;  // NHWC [Nimg][Hs][Ws][Cs]
    const void *wpk;  // [Ngemm][ntaps][Cs]
    void *out;        // NHWC [Nimg][Ho][Wo][Co]
    int Nimg, Hs, Ws, Cs;
    int Mi, Mj, M;
    int mult_h, add_h, mult_w, add_w;
    int ntaps, Ktot;
    int Ngemm;
    int Ho, Wo, Co;
    int osh, oa, osw, ob;
    int accumulate;
    int vec_out;  // set by launch_igemm: output rows are 16-byte granular, vector epilogue
    unsigned src_bytes, wpk_bytes;  // sizes of src and wpk (both below 4 GiB: buffer addressing)
    // Optional per-channel partial sums of the STORED output for a following batch-norm: stats[0][r][n] = sum and
    // stats[1][r][n] = sum of squares over the r-th disjoint share of the rows, r < stats_rows.  Only set when
    // igemm_stats_rows() named the row count for exactly this launch.
    float *stats;
    int stats_rows;
    // Forward with the producing batch-norm and ReLU applied to the input on load: src holds the RAW output of the
    // previous convolution and the kernel multiplies relu(act[c]*src + act[Cs + c]) (zero padding stays zero).  Only
    // kernels for which igemm_act_fused() says yes take it; nullptr otherwise.
    const float *act;
    // Backward-data of a stride-2 layer whose taps all fall into residue class (0, 0): the launch for that class also
    // writes zeros to the other (up to three) pixels of each row's 2x2 output cell.  Only the short-reduction kernel
    // honours it: set it only after conv_pw_applicable() said yes for these arguments.
    int zero_cell;
    // Grouped convolution (groups > 1; 0 or 1 = plain): the launch computes `groups` independent problems of the
    // shape above.  Group g reads channels [g*Cs, (g+1)*Cs) of source pixels that are src_ld channels apart, the filter
    // rows [g*Ngemm, (g+1)*Ngemm) of wpk, and writes columns [g*Ngemm, (g+1)*Ngemm) of the Co-channel output pixels.
    // Only the generic kernel runs such launches; src_ld is ignored (taken as Cs) for plain ones.
    int groups, src_ld;
    short off_h[kMaxTaps];
    short off_w[kMaxTaps];
};
int launch_igemm(int dtype, const IgemmArgs &a, hipStream_t stream);
// True if the kernel launch_igemm picks for these arguments applies IgemmArgs::act while it stages its input.
bool igemm_act_fused(int dtype, const IgemmArgs &a);
// Rows of partial sums the kernel launch_igemm would pick writes from its epilogue; 0 if that kernel has no
// statistics epilogue (the caller then runs a separate reduction pass).  Host only, depends on the shape alone.
int igemm_stats_rows(int dtype, const IgemmArgs &a);
// bf16 large-tile kernel for wide layers (channel counts that are multiples of 64, enough tiles to fill the chip)
bool igemm_big_applicable(int dtype, const IgemmArgs &a);
int launch_igemm_big(const IgemmArgs &a, hipStream_t stream);
int igemm_big_stats_rows(const IgemmArgs &a);
// the residue classes of one strided backward-data pass (2..4 argument sets on the same tensors) in one launch
bool igemm_big_multi_applicable(int dtype, const IgemmArgs *a, int count);
int launch_igemm_big_multi(const IgemmArgs *a, int count, hipStream_t stream);
// bf16 layers with one, two or four taps and at most 256 reduction indices (memory-bound: filter resident in LDS,
// pixels loaded straight into MFMA operand registers)
bool conv_pw_applicable(int dtype, const IgemmArgs &a);
int launch_conv_pw(const IgemmArgs &a, hipStream_t stream);
int conv_pw_stats_rows(const IgemmArgs &a);
// bf16 3x3 stride-1 64->64 special case (filter resident in LDS, input tile staged once with halo)
bool halo64_applicable(int dtype, const IgemmArgs &a);
int launch_halo64(const IgemmArgs &a, hipStream_t stream);
int halo64_stats_rows(const IgemmArgs &a);
// bf16 3x3 stride-1 layers with 128..512 input channels (input rows with halo staged once, filter streamed from L2
// into MFMA operand registers)
bool halo_wide_applicable(int dtype, const IgemmArgs &a);
int launch_halo_wide(const IgemmArgs &a, hipStream_t stream);
int halo_wide_stats_rows(const IgemmArgs &a);
// forward of a 3x3 stride-2 pad-1 layer with 128 or 256 input channels: the same kernel on four parity planes of x
bool halo_wide_fwd_s2_applicable(int dtype, const IgemmArgs &a);
int halo_wide_fwd_s2_stats_rows(const IgemmArgs &a);
int launch_halo_wide_fwd_s2(const IgemmArgs &a, hipStream_t stream);
// the four residue classes of the backward-data pass of a bf16 3x3 stride-2 64 -> 64 layer in one launch of the
// filter-stationary kernel (conv_fs64_s2.hip)
bool fs64_dgrad_s2_applicable(int dtype, const IgemmArgs *a, int count);
int launch_fs64_dgrad_s2(const IgemmArgs *a, int count, hipStream_t stream);
// forward of the same layer (stride 2 as four parity planes of the input), same file
bool fs64_fwd_s2_applicable(int dtype, const IgemmArgs &a);
int fs64_fwd_s2_stats_rows(const IgemmArgs &a);
int launch_fs64_fwd_s2(const IgemmArgs &a, hipStream_t stream);
// the residue classes of one strided backward-data pass of such a layer in one launch, sharing the staged tiles
bool halo_wide_multi_applicable(int dtype, const IgemmArgs *a, int count);
int launch_halo_wide_multi(const IgemmArgs *a, int count, hipStream_t stream);
// fp32 sibling (filter streamed one tap at a time through LDS)
bool halo64_f32_applicable(int dtype, const IgemmArgs &a);
int launch_halo64_f32(const IgemmArgs &a, hipStream_t stream);
int halo64_f32_stats_rows(const IgemmArgs &a);

// layers with at most four channels on one side (the 3-channel stride-1 image stem): direct kernels, no MFMA
bool tiny_src_applicable(int dtype, const IgemmArgs &a);    // few source channels (forward)
int launch_tiny_src(int dtype, const IgemmArgs &a, hipStream_t stream);
bool tiny_out_applicable(int dtype, const IgemmArgs &a);    // few output channels (backward-data)
int launch_tiny_out(int dtype, const IgemmArgs &a, hipStream_t stream);
// depthwise layers (grouped launches with one channel per group on both sides, channel count a multiple of the vector
// width): direct kernels bound by memory bandwidth, no MFMA
bool depthwise_applicable(int dtype, const IgemmArgs &a);
int launch_depthwise(int dtype, const IgemmArgs &a, hipStream_t stream);

// ------------------------------------------------------------------ wgrad
// part[split][k][t][c] = sum over the split's share of rows l = (img, p, q) of
//   dy[img][p][q][k] * x[img][p*sh - ph + off_h[t]][q*sw - pw + off_w[t]][c]
struct WgradArgs {
    const void *x;   // NHWC [Nimg][H][W][C]
    const void *dy;  // NHWC [Nimg][P][Q][K]
    float *part;     // [splits][K][ntaps*C]
    int Nimg, H, W, C, P, Q, K;
    int sh, sw, ph, pw;
    int ntaps;
    int L;           // Nimg*P*Q
    int rows_per_split;  // multiple of the kernel's BK
    int splits;
    // Grouped convolution (groups > 1; 0 or 1 = plain): C and K are the channel counts of ONE group, pixels of x are ldx
    // channels apart and pixels of dy ldy channels; group g reads the channel runs [g*C, (g+1)*C) and [g*K, (g+1)*K)
    // and writes rows [g*K, (g+1)*K) of part[split][groups*K][ntaps*C].  Only the generic kernel runs such launches;
    // ldx and ldy are ignored (taken as C and K) for plain ones.
    int groups, ldx, ldy;
    // nullptr, or [2][C]: x holds the RAW output of the producing convolution and the kernel uses
    // relu(act[c]*x + act[C + c]); only where wgrad_halo64_act_fused() says yes
    const float *act;
    short off_h[kMaxTaps];
    short off_w[kMaxTaps];
};
int wgrad_rows_per_split(int dtype, int L, int K, int ntapsC, int *splits);
int launch_wgrad(int dtype, const WgradArgs &a, hipStream_t stream);
// 3x3 stride-1 64->64 special case: one [K][taps][C] partial per block, `partials` of them
bool wgrad_halo64_applicable(int dtype, const WgradArgs &a);
int wgrad_halo64_partials(int dtype, const WgradArgs &a, int *chunks_per_block);
int launch_wgrad_halo64(int dtype, const WgradArgs &a, hipStream_t stream);
bool wgrad_halo64_act_fused(int dtype, const WgradArgs &a);
// wide bf16 layers (C, K multiples of 64, long reduction): large tiles, about one block per CU
bool wgrad_wide_applicable(int dtype, const WgradArgs &a);
int wgrad_wide_rows_per_split(const WgradArgs &a, int *splits);
int launch_wgrad_wide(const WgradArgs &a, hipStream_t stream);
// at most four input channels: partial sums in the layout of the generic kernel
bool tiny_wgrad_applicable(int dtype, const WgradArgs &a);
int launch_tiny_wgrad(int dtype, const WgradArgs &a, hipStream_t stream);
// depthwise layers: partial sums in the layout of the generic kernel's grouped launch
bool depthwise_wgrad_applicable(int dtype, const WgradArgs &a);
int launch_depthwise_wgrad(int dtype, const WgradArgs &a, hipStream_t stream);
// dw[k*sk + t*st + c*sc] (=|+=) sum_s part[s][k][t][c], fixed order.
int launch_wgrad_reduce(const float *part, float *dw, int splits, int K, int ntaps, int C,
                        long sk, long st, long sc, int accumulate, hipStream_t stream);

// ------------------------------------------------------------------ image stem
// Stride-2 odd square filter with "same" padding on at most 4 input channels and even H, W: all three
// passes run on a space-to-depth copy of the image (16 channels, stride 1).  `ws` must hold
// stem_workspace_bytes(g, pass) bytes.
bool stem_applicable(const ConvGeo &g);
size_t stem_workspace_bytes(const ConvGeo &g, int pass);
// stats / stats_rows: as in IgemmArgs (nullptr: none); *y_nhwc receives the NHWC result (y itself, or its workspace
// copy for NCHW descriptors)
int stem_fwd(const ConvGeo &g, const void *x, const void *w, void *y, char *ws, float *stats, int stats_rows,
             void **y_nhwc, hipStream_t stream);
int stem_stats_rows(const ConvGeo &g);
int stem_dgrad(const ConvGeo &g, const void *dy, const void *w, void *dx, int accumulate, char *ws, hipStream_t stream);
int stem_wgrad(const ConvGeo &g, const void *x, const void *dy, float *dw, int accumulate, char *ws, hipStream_t stream);

// 7x7 stem (4x4 coarse taps), bf16, 64 output channels: forward / backward-data on the space-to-depth grid
bool stem_halo_applicable(int dtype, int U, int K, int Nimg, int H, int W);
int launch_stem_halo(int backward, const void *src, const void *wpk, void *out, int Nimg, int H, int W, float *stats,
                     int stats_rows, hipStream_t stream);
int stem_halo_stats_rows(int Nimg, int H, int W);

// ------------------------------------------------------------------ layout helpers
// dst NHWC <- src NCHW (plain copy).
int launch_nchw_to_nhwc(int dtype, const void *src, void *dst, int N, int C, int H, int W,
                        hipStream_t stream);
// dst NCHW (=|+=) src NHWC.
int launch_nhwc_to_nchw(int dtype, const void *src, void *dst, int N, int C, int H, int W,
                        int accumulate, hipStream_t stream);
// out[n][t][c] = w[n*sn + tap_off[t] + c*sc] for n < Nn, t < ntaps, c < Cs.
int launch_pack_filter(int dtype, const void *w, void *out, int Nn, int ntaps, int Cs, long sn,
                       long sc, const int *tap_off_host, hipStream_t stream);
// The same for up to four tap subsets of one filter in one launch: out[k][n][t][c] with ntaps[k] taps tap_off_host[k][.].
int launch_pack_filters(int dtype, int count, const void *w, void *const *out, int Nn, const int *ntaps, int Cs, long sn,
                        long sc, const int (*tap_off_host)[kMaxTaps], hipStream_t stream);
// The same for `groups` filters that lie w_gstep elements apart in w: out[k][g][n][t][c] = w[g*w_gstep + n*sn + ...].
int launch_pack_filters_grouped(int dtype, int count, const void *w, void *const *out, int Nn, const int *ntaps, int Cs,
                                long sn, long sc, const int (*tap_off_host)[kMaxTaps], int groups, long w_gstep,
                                hipStream_t stream);

// out[img][i*osh + oa][j*osw + ob][0..Co) = 0 for i < Mi, j < Mj (NHWC).
int launch_zero_class(int dtype, void *out, int Nimg, int Ho, int Wo, int Co, int Mi, int Mj, int osh, int oa, int osw,
                      int ob, hipStream_t stream);

// ------------------------------------------------------------------ batch-norm, pooling
int bn_partial_blocks(const nsk_bn_desc_t &d);
size_t bn_mask_bytes(const nsk_bn_desc_t &d);
int launch_bn_fwd(const nsk_bn_desc_t &d, const void *x, const void *residual, const float *gamma,
                  const float *beta, void *out, float *save_mean, float *save_invstd,
                  float *running_mean, float *running_var, void *ws, unsigned char *relu_mask, const float *stats,
                  int stats_rows, hipStream_t stream);
int bn_stats_rows(const nsk_bn_desc_t &d);
int launch_bn_stats(const nsk_bn_desc_t &d, const void *x, float *stats, hipStream_t stream);
int launch_bn_bwd(const nsk_bn_desc_t &d, const void *x, const void *out, const void *dout,
                  const float *gamma, const float *save_mean, const float *save_invstd, void *dx,
                  void *dres, float *dgamma, float *dbeta, void *ws, const unsigned char *relu_mask,
                  hipStream_t stream, const float *act = nullptr);
// The normalised activation applied by its consumers on load (scale and shift per channel: coeffs = [2][C] floats)
bool bn_act_supported(const nsk_bn_desc_t &d);
int launch_bn_coeffs(const nsk_bn_desc_t &d, const float *gamma, const float *beta, const float *stats, int stats_rows,
                     float *save_mean, float *save_invstd, float *running_mean, float *running_var, float *coeffs,
                     void *ws, hipStream_t stream);
int launch_bn_act(const nsk_bn_desc_t &d, const void *x, const float *coeffs, void *out, hipStream_t stream);
int launch_maxpool_fwd(const nsk_pool_desc_t &d, int P, int Q, const void *x, void *y,
                       signed char *idx, hipStream_t stream);
int launch_maxpool_bwd(const nsk_pool_desc_t &d, int P, int Q, const void *dy,
                       const signed char *idx, void *dx, hipStream_t stream);

}  // namespace nsk

// Depthwise convolution (a grouped convolution with one input and one output channel per group; the grouped entry
// points of the library, not one of the paper's workloads): y[n][p][q][c] = sum over taps of x[n][h][w][c] * w[c][tap],
// and its neighbours with two, four or (bf16) eight channels per group on both sides (template parameter CG), where an output channel
// sums over the CG input channels of its group.
// The contraction over channels is absent or tiny, so nothing here is GEMM-shaped: every pass reads each activation once from
// HBM (the taps' re-reads hit the caches), does ntaps multiply-adds per element on the vector ALUs and is bound by
// memory bandwidth.  NHWC puts the channels of a pixel side by side, so a lane owns one 16-byte vector of channels
// and consecutive lanes read consecutive addresses.
//
//  - forward / backward-data: the argument set of the implicit-GEMM kernels (gather taps around a base pixel, store
//    to a strided output grid) with Cs = Ngemm = 1; a lane computes DW_PIX consecutive output pixels of its channel
//    vector, the filter lives transposed ([tap][channel], float) in LDS.
//  - backward-weight: dw[c][tap] = sum over output pixels of dy * shifted x.  A block owns up to 16 channel vectors
//    and one split of the pixels; its pixel lanes stride through the split with the per-tap sums in registers and are
//    combined through LDS in a fixed order.  The partial sums land in the layout of the generic split kernel, so the
//    same deterministic reduction finishes the job.
#include <stdlib.h>

#include "nsk_internal.h"

namespace nsk {
namespace {

constexpr int DW_PIX = 4;          // output pixels per lane (forward / backward-data)
constexpr int DW_ROUND = 3;        // taps whose loads are issued together
constexpr int DW_LDS_MAX = 48 << 10;  // bytes of LDS the transposed filter may take
constexpr int DW_CVB = 16;         // channel vectors per backward-weight block

template <typename T> struct DTraits;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <> struct DTraits<float> {
    static constexpr int VEC = 4;
    typedef f32x4 Vec;
};
template <> struct DTraits<bf16_t> {
    static constexpr int VEC = 8;
    typedef bf16x8 Vec;
};

typedef bf16_t bf16x2 __attribute__((ext_vector_type(2)));

// acc += x . w over the two bf16 halves of a dword: one instruction per product pair, no conversion to float.  Only used
// where both halves belong to the same group (two or more channels per group).
__device__ inline float dot2(unsigned x, unsigned w, float acc)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, x), __builtin_bit_cast(bf16x2, w), acc, false);
}

// LDS words per (tap, output channel): floats w[k][t][0..CG) for fp32; for bf16 dwords of two filter values each
// (CG = 1: the one filter value as a float).
template <typename T, int CG> constexpr int lds_words() { return sizeof(T) == 4 ? CG : (CG + 1) / 2; }

// acc[e] += sum over the CG input channels of output channel e's group of x * w, for the VEC output channels of one
// channel vector; xv = the pixel's vector as loaded, wv = the LDS words of these output channels for one tap.
template <typename T, int CG>
__device__ inline void mac_vec(float (&acc)[DTraits<T>::VEC], const u32x4 &xv,
                               const unsigned (&wv)[DTraits<T>::VEC * lds_words<T, CG>()])
{
    constexpr int VEC = DTraits<T>::VEC, WPK = lds_words<T, CG>();
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        if constexpr (sizeof(T) == 4) {
            // the group's input channels are words (e / CG) * CG .. of the vector
#pragma unroll
            for (int cl = 0; cl < CG; ++cl)
                acc[e] += __uint_as_float(xv[(e / CG) * CG + cl]) * __uint_as_float(wv[e * CG + cl]);
        } else if constexpr (CG == 1) {
            // plain multiply-add on the channel's own half of the dword: a two-element dot product with a zero weight
            // in the other half would let an infinity in the NEIGHBOURING channel turn this one into NaN (the dot
            // product was 15% faster at 128 channels on 56x56 images, which this property is worth)
            const unsigned d = xv[e / 2];
            acc[e] += __uint_as_float((e & 1) ? (d & 0xFFFF0000u) : (d << 16)) * __uint_as_float(wv[e]);
        } else {
            // the group's input channels are dwords (e / CG) * (CG / 2) .. of the vector
#pragma unroll
            for (int j = 0; j < WPK; ++j) acc[e] = dot2(xv[(e / CG) * WPK + j], wv[e * WPK + j], acc[e]);
        }
    }
}

// The filter of a launch, as the kernels keep it in LDS: wL[(tap * C + channel) * WPK + word].
template <typename T, int CG> __device__ inline void stage_filter(const IgemmArgs &a, unsigned *wL, int C)
{
    constexpr int WPK = lds_words<T, CG>();
    const int tid = threadIdx.x, ntaps = a.ntaps;
    if constexpr (sizeof(T) == 4) {
        const float *__restrict__ wpk = (const float *)a.wpk;      // [C][ntaps][CG]
        for (int i = tid; i < ntaps * C * CG; i += 256) {
            const int cl = i % CG, r = i / CG;
            const int c = r / ntaps, t = r - c * ntaps;
            wL[(t * C + c) * CG + cl] = __float_as_uint(wpk[i]);
        }
    } else {
        const unsigned short *__restrict__ wpk = (const unsigned short *)a.wpk;
        for (int i = tid; i < ntaps * C * WPK; i += 256) {
            const int j = i % WPK, r = i / WPK;
            const int c = r / ntaps, t = r - c * ntaps;
            unsigned v;
            if (CG == 1) {
                v = (unsigned)wpk[r] << 16;   // the filter value as a float
            } else {
                const unsigned short *q = wpk + (long)r * CG + 2 * j;
                v = (unsigned)q[0] | ((unsigned)q[1] << 16);
            }
            wL[(t * C + c) * WPK + j] = v;
        }
    }
}

template <typename T, int CG>
__global__ __launch_bounds__(256) void depthwise_kernel(const IgemmArgs a, const int iters)
{
    typedef typename DTraits<T>::Vec Vec;
    constexpr int VEC = DTraits<T>::VEC;
    constexpr int WPK = lds_words<T, CG>();
    static_assert(VEC % CG == 0, "a channel vector holds whole groups");
    extern __shared__ __attribute__((aligned(16))) unsigned wL[];   // [ntaps][C][WPK]
    __shared__ short s_offh[kMaxTaps], s_offw[kMaxTaps];
    const int tid = threadIdx.x;
    const int C = a.groups * CG, CV = C / VEC, ntaps = a.ntaps;
    T *__restrict__ out = (T *)a.out;
    stage_filter<T, CG>(a, wL, C);
    if (tid < kMaxTaps) {
        s_offh[tid] = a.off_h[tid];
        s_offw[tid] = a.off_w[tid];
    }
    __syncthreads();

    // Loads go through a buffer descriptor: an offset of ~0 is out of range and returns zeros, so a tap outside the
    // image costs no branch and the loads of a round of taps are all in flight together.
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.src, 0, a.src_bytes, 0x00020000);
    // a block takes `iters` consecutive runs of 256 (pixel group, channel vector) pairs: the staged filter serves them all
    for (int it = 0; it < iters; ++it) {
    const long f = ((long)blockIdx.x * iters + it) * 256 + tid;
    const int cv = (int)(f % CV);
    const long slot = f / CV;
    if (slot * DW_PIX >= a.M) break;
    const int c0 = cv * VEC;
    bool ok[DW_PIX];
    int bh[DW_PIX], bw[DW_PIX];
    unsigned base[DW_PIX];
    long out_off[DW_PIX];
    float acc[DW_PIX][VEC];
    const int per_img = a.Mi * a.Mj;
#pragma unroll
    for (int u = 0; u < DW_PIX; ++u) {
        const long m = slot * DW_PIX + u;
        ok[u] = m < a.M;
        const int mm = ok[u] ? (int)m : 0;
        const int img = mm / per_img;
        const int rem = mm - img * per_img;
        const int i = rem / a.Mj;
        const int j = rem - i * a.Mj;
        bh[u] = i * a.mult_h + a.add_h;
        bw[u] = j * a.mult_w + a.add_w;
        base[u] = (unsigned)(((((long)img * a.Hs + bh[u]) * a.Ws + bw[u]) * C + c0) * (long)sizeof(T));
        out_off[u] = (((long)img * a.Ho + (i * a.osh + a.oa)) * a.Wo + (j * a.osw + a.ob)) * C + c0;
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[u][e] = 0.f;
        if (a.accumulate && ok[u]) {   // start from the old values: the sum is rounded to the storage type once
            const Vec old = *(const Vec *)(out + out_off[u]);
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[u][e] = (float)old[e];
        }
    }
    for (int t0 = 0; t0 < ntaps; t0 += DW_ROUND) {
        u32x4 xv[DW_ROUND][DW_PIX];
        int tt[DW_ROUND];
#pragma unroll
        for (int k = 0; k < DW_ROUND; ++k) {
            const bool tap_ok = t0 + k < ntaps;
            tt[k] = tap_ok ? t0 + k : ntaps - 1;
            const int oh = s_offh[tt[k]], ow = s_offw[tt[k]];
            const unsigned delta = (unsigned)((oh * a.Ws + ow) * C * (int)sizeof(T));
#pragma unroll
            for (int u = 0; u < DW_PIX; ++u) {
                const int h = bh[u] + oh, w = bw[u] + ow;
                const bool in = tap_ok && ok[u] && (unsigned)h < (unsigned)a.Hs && (unsigned)w < (unsigned)a.Ws;
                xv[k][u] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, in ? base[u] + delta : ~0u, 0, 0));
            }
        }
#pragma unroll
        for (int k = 0; k < DW_ROUND; ++k) {
            unsigned wv[VEC * WPK];
#pragma unroll
            for (int e = 0; e < VEC * WPK; e += 4) {
                const u32x4 q = *(const u32x4 *)&wL[(tt[k] * C + c0) * WPK + e];
                wv[e] = q[0]; wv[e + 1] = q[1]; wv[e + 2] = q[2]; wv[e + 3] = q[3];
            }
#pragma unroll
            for (int u = 0; u < DW_PIX; ++u) mac_vec<T, CG>(acc[u], xv[k][u], wv);
        }
    }
#pragma unroll
    for (int u = 0; u < DW_PIX; ++u) {
        if (!ok[u]) continue;
        Vec o;
#pragma unroll
        for (int e = 0; e < VEC; ++e) o[e] = (T)acc[u][e];
        __builtin_nontemporal_store(o, (Vec *)(out + out_off[u]));   // the output is not read again: keep the caches for the input
    }
    }
}

// Taps that form a grid of up to 8 rows x S consecutive columns, on output columns that map to consecutive source
// columns (stride 1 along the width): `tap[rr * S + ss]` is the tap at row offset row_off[rr], column offset w_min + ss.
struct RowPlan {
    int R, w_min;
    short row_off[8];
    unsigned char tap[kMaxTaps];
};

// The same computation for such launches with the DW_PIX outputs of a lane side by side in one output row: a source row
// is loaded once for all of them (S + DW_PIX - 1 vectors instead of S * DW_PIX), which halves the traffic between the
// caches and the CUs for a 3x3 filter.
template <typename T, int CG, int S>
__global__ __launch_bounds__(256) void depthwise_row_kernel(const IgemmArgs a, const RowPlan rp, const int iters)
{
    typedef typename DTraits<T>::Vec Vec;
    constexpr int VEC = DTraits<T>::VEC;
    constexpr int WPK = lds_words<T, CG>();
    constexpr int NCOL = S + DW_PIX - 1;
    extern __shared__ __attribute__((aligned(16))) unsigned wL[];   // [ntaps][C][WPK]
    const int tid = threadIdx.x;
    const int C = a.groups * CG, CV = C / VEC;
    T *__restrict__ out = (T *)a.out;
    stage_filter<T, CG>(a, wL, C);
    __syncthreads();
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.src, 0, a.src_bytes, 0x00020000);
    const int JG = (a.Mj + DW_PIX - 1) / DW_PIX;      // lanes per output row and channel vector
    const long slots = (long)a.Nimg * a.Mi * JG;
    for (int it = 0; it < iters; ++it) {
        const long f = ((long)blockIdx.x * iters + it) * 256 + tid;
        const int cv = (int)(f % CV);
        const long slot = f / CV;
        if (slot >= slots) break;
        const int c0 = cv * VEC;
        const int jg = (int)(slot % JG);
        const long r = slot / JG;
        const int i = (int)(r % a.Mi);
        const int img = (int)(r / a.Mi);
        const int j0 = jg * DW_PIX;
        const int bh = i * a.mult_h + a.add_h, bw = j0 + a.add_w + rp.w_min;   // first source column of the lane
        const long out_off = (((long)img * a.Ho + (i * a.osh + a.oa)) * a.Wo + (j0 * a.osw + a.ob)) * C + c0;
        const long out_step = (long)a.osw * C;
        float acc[DW_PIX][VEC];
#pragma unroll
        for (int u = 0; u < DW_PIX; ++u) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[u][e] = 0.f;
            if (a.accumulate && j0 + u < a.Mj) {   // start from the old values: the sum is rounded to the storage type once
                const Vec old = *(const Vec *)(out + out_off + u * out_step);
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[u][e] = (float)old[e];
            }
        }
        for (int rr = 0; rr < rp.R; ++rr) {
            const int h = bh + rp.row_off[rr];
            const bool row_ok = (unsigned)h < (unsigned)a.Hs;
            const unsigned base = (unsigned)(((((long)img * a.Hs + h) * a.Ws + bw) * C + c0) * (long)sizeof(T));
            u32x4 xv[NCOL];
#pragma unroll
            for (int k = 0; k < NCOL; ++k) {
                const bool in = row_ok && (unsigned)(bw + k) < (unsigned)a.Ws;
                xv[k] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(
                                                      rsrc, in ? base + (unsigned)(k * C * (int)sizeof(T)) : ~0u, 0, 0));
            }
#pragma unroll
            for (int ss = 0; ss < S; ++ss) {
                const int t = rp.tap[rr * S + ss];
                unsigned wv[VEC * WPK];
#pragma unroll
                for (int e = 0; e < VEC * WPK; e += 4) {
                    const u32x4 q = *(const u32x4 *)&wL[(t * C + c0) * WPK + e];
                    wv[e] = q[0]; wv[e + 1] = q[1]; wv[e + 2] = q[2]; wv[e + 3] = q[3];
                }
#pragma unroll
                for (int u = 0; u < DW_PIX; ++u) mac_vec<T, CG>(acc[u], xv[u + ss], wv);
            }
        }
#pragma unroll
        for (int u = 0; u < DW_PIX; ++u) {
            if (j0 + u >= a.Mj) continue;
            Vec o;
#pragma unroll
            for (int e = 0; e < VEC; ++e) o[e] = (T)acc[u][e];
            __builtin_nontemporal_store(o, (Vec *)(out + out_off + u * out_step));
        }
    }
}

// Fills the plan if the launch's taps form such a grid (see RowPlan) with S = 3, 5 or 7 columns.
bool row_plan(const IgemmArgs &a, RowPlan *rp)
{
    if (a.mult_w != 1 || a.ntaps < 3) return false;
    int w_min = a.off_w[0], w_max = a.off_w[0];
    for (int t = 1; t < a.ntaps; ++t) {
        if (a.off_w[t] < w_min) w_min = a.off_w[t];
        if (a.off_w[t] > w_max) w_max = a.off_w[t];
    }
    const int S = w_max - w_min + 1;
    if ((S != 3 && S != 5 && S != 7) || a.ntaps % S != 0 || a.ntaps / S > 8) return false;
    rp->R = 0;
    rp->w_min = w_min;
    bool seen[kMaxTaps] = {};
    for (int t = 0; t < a.ntaps; ++t) {
        int rr = 0;
        while (rr < rp->R && rp->row_off[rr] != a.off_h[t]) ++rr;
        if (rr == rp->R) {
            if (rp->R == a.ntaps / S) return false;   // more distinct rows than a full grid has
            rp->row_off[rp->R++] = a.off_h[t];
        }
        const int cell = rr * S + (a.off_w[t] - w_min);
        if (seen[cell]) return false;
        seen[cell] = true;
        rp->tap[cell] = (unsigned char)t;
    }
    return rp->R * S == a.ntaps;   // every cell seen exactly once
}

// The transposed arrangement: taps in a grid of R consecutive ROWS (height stride 1) x up to 8 columns, and the DW_PIX
// outputs of a lane stacked in one output COLUMN.  Consecutive lanes then hold consecutive channel vectors of consecutive
// pixels of a row, so every load of a wavefront covers one contiguous kilobyte (the row-sharing kernel's loads cover four
// pieces a kilobyte apart), and a source column piece is still loaded once for all of a lane's outputs.
// `tap[ss * R + rr]` is the tap at column offset col_off[ss], row offset h_min + rr.
struct ColPlan {
    int S, h_min;
    short col_off[8];
    unsigned char tap[kMaxTaps];
};

template <typename T, int CG, int R>
__global__ __launch_bounds__(256) void depthwise_col_kernel(const IgemmArgs a, const ColPlan cp, const int iters)
{
    typedef typename DTraits<T>::Vec Vec;
    constexpr int VEC = DTraits<T>::VEC;
    constexpr int WPK = lds_words<T, CG>();
    constexpr int NROW = R + DW_PIX - 1;
    extern __shared__ __attribute__((aligned(16))) unsigned wL[];   // [ntaps][C][WPK]
    const int tid = threadIdx.x;
    const int C = a.groups * CG, CV = C / VEC;
    T *__restrict__ out = (T *)a.out;
    stage_filter<T, CG>(a, wL, C);
    __syncthreads();
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.src, 0, a.src_bytes, 0x00020000);
    const int IG = (a.Mi + DW_PIX - 1) / DW_PIX;      // groups of output rows
    const long slots = (long)a.Nimg * IG * a.Mj;       // (image, row group, column): the column runs fastest
    for (int it = 0; it < iters; ++it) {
        const long f = ((long)blockIdx.x * iters + it) * 256 + tid;
        const int cv = (int)(f % CV);
        const long slot = f / CV;
        if (slot >= slots) break;
        const int c0 = cv * VEC;
        const int j = (int)(slot % a.Mj);
        const long r = slot / a.Mj;
        const int ig = (int)(r % IG);
        const int img = (int)(r / IG);
        const int i0 = ig * DW_PIX;
        const int bh = i0 + a.add_h + cp.h_min, bw = j * a.mult_w + a.add_w;   // first source row of the lane
        const long out_off = (((long)img * a.Ho + (i0 * a.osh + a.oa)) * a.Wo + (j * a.osw + a.ob)) * C + c0;
        const long out_step = (long)a.osh * a.Wo * C;
        float acc[DW_PIX][VEC];
#pragma unroll
        for (int u = 0; u < DW_PIX; ++u) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[u][e] = 0.f;
            if (a.accumulate && i0 + u < a.Mi) {   // start from the old values: the sum is rounded to the storage type once
                const Vec old = *(const Vec *)(out + out_off + u * out_step);
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[u][e] = (float)old[e];
            }
        }
        for (int ss = 0; ss < cp.S; ++ss) {
            const int w = bw + cp.col_off[ss];
            const bool col_ok = (unsigned)w < (unsigned)a.Ws;
            const unsigned base = (unsigned)(((((long)img * a.Hs + bh) * a.Ws + w) * C + c0) * (long)sizeof(T));
            u32x4 xv[NROW];
#pragma unroll
            for (int k = 0; k < NROW; ++k) {
                const bool in = col_ok && (unsigned)(bh + k) < (unsigned)a.Hs;
                xv[k] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(
                                                      rsrc, in ? base + (unsigned)(k * a.Ws * C * (int)sizeof(T)) : ~0u, 0, 0));
            }
#pragma unroll
            for (int rr = 0; rr < R; ++rr) {
                const int t = cp.tap[ss * R + rr];
                unsigned wv[VEC * WPK];
#pragma unroll
                for (int e = 0; e < VEC * WPK; e += 4) {
                    const u32x4 q = *(const u32x4 *)&wL[(t * C + c0) * WPK + e];
                    wv[e] = q[0]; wv[e + 1] = q[1]; wv[e + 2] = q[2]; wv[e + 3] = q[3];
                }
#pragma unroll
                for (int u = 0; u < DW_PIX; ++u) mac_vec<T, CG>(acc[u], xv[u + rr], wv);
            }
        }
#pragma unroll
        for (int u = 0; u < DW_PIX; ++u) {
            if (i0 + u >= a.Mi) continue;
            Vec o;
#pragma unroll
            for (int e = 0; e < VEC; ++e) o[e] = (T)acc[u][e];
            __builtin_nontemporal_store(o, (Vec *)(out + out_off + u * out_step));
        }
    }
}

// Fills the plan if the launch's taps form such a grid (see ColPlan) with R = 3, 5 or 7 rows.
bool col_plan(const IgemmArgs &a, ColPlan *cp)
{
    if (a.mult_h != 1 || a.ntaps < 3) return false;
    int h_min = a.off_h[0], h_max = a.off_h[0];
    for (int t = 1; t < a.ntaps; ++t) {
        if (a.off_h[t] < h_min) h_min = a.off_h[t];
        if (a.off_h[t] > h_max) h_max = a.off_h[t];
    }
    const int R = h_max - h_min + 1;
    if ((R != 3 && R != 5 && R != 7) || a.ntaps % R != 0 || a.ntaps / R > 8) return false;
    cp->S = 0;
    cp->h_min = h_min;
    bool seen[kMaxTaps] = {};
    for (int t = 0; t < a.ntaps; ++t) {
        int ss = 0;
        while (ss < cp->S && cp->col_off[ss] != a.off_w[t]) ++ss;
        if (ss == cp->S) {
            if (cp->S == a.ntaps / R) return false;   // more distinct columns than a full grid has
            cp->col_off[cp->S++] = a.off_w[t];
        }
        const int cell = ss * R + (a.off_h[t] - h_min);
        if (seen[cell]) return false;
        seen[cell] = true;
        cp->tap[cell] = (unsigned char)t;
    }
    return cp->S * R == a.ntaps;   // every cell seen exactly once
}

// Taps per register chunk of the backward-weight kernel: a lane keeps taps x VEC x CG sums.
template <int CG> constexpr int wgrad_taps() { return CG == 1 ? 9 : (CG == 2 ? 5 : (CG == 4 ? 3 : 1)); }

template <typename T, int CG>
__global__ __launch_bounds__(256) void depthwise_wgrad_kernel(const WgradArgs a)
{
    typedef typename DTraits<T>::Vec Vec;
    constexpr int VEC = DTraits<T>::VEC;
    constexpr int TC = wgrad_taps<CG>();
    __shared__ float red[256 * VEC];
    __shared__ short s_offh[kMaxTaps], s_offw[kMaxTaps];
    const int tid = threadIdx.x;
    const int C = a.groups * CG, CV = C / VEC;
    const int cvb = min(CV - (int)blockIdx.x * DW_CVB, DW_CVB);   // channel vectors of this block (>= 1)
    const int PL = 256 / cvb;                                     // pixel lanes
    const int cvl = tid % cvb, pl = tid / cvb;
    const bool active = pl < PL;
    const int c0 = (blockIdx.x * DW_CVB + cvl) * VEC;
    const int split = blockIdx.y;
    const T *__restrict__ dy = (const T *)a.dy;
    // x through a buffer descriptor (an offset of ~0 returns zeros): taps outside the image cost no branch
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)a.x, 0, (unsigned)((long)a.Nimg * a.H * a.W * C * (long)sizeof(T)), 0x00020000);
    if (tid < kMaxTaps) {
        s_offh[tid] = a.off_h[tid];
        s_offw[tid] = a.off_w[tid];
    }
    __syncthreads();
    const int l_begin = split * a.rows_per_split;
    const int l_end = min(a.L, l_begin + a.rows_per_split);
    const int pq = a.P * a.Q;
    float *__restrict__ part = a.part + (long)split * C * a.ntaps * CG;   // [C][ntaps][CG]

    for (int t0 = 0; t0 < a.ntaps; t0 += TC) {
        float acc[TC][VEC][CG];
#pragma unroll
        for (int tt = 0; tt < TC; ++tt)
#pragma unroll
            for (int e = 0; e < VEC; ++e)
#pragma unroll
                for (int cl = 0; cl < CG; ++cl) acc[tt][e][cl] = 0.f;
        if (active)
#pragma unroll 2
            for (int l = l_begin + pl; l < l_end; l += PL) {
                const int img = l / pq;
                const int rem = l - img * pq;
                const int p = rem / a.Q;
                const int q = rem - p * a.Q;
                const Vec dv = *(const Vec *)(dy + (long)l * C + c0);
                const int h0 = p * a.sh - a.ph, w0 = q * a.sw - a.pw;
                const unsigned base = (unsigned)(((((long)img * a.H + h0) * a.W + w0) * C + c0) * (long)sizeof(T));
                Vec xv[TC];
#pragma unroll
                for (int tt = 0; tt < TC; ++tt) {
                    const int t = min(t0 + tt, a.ntaps - 1);
                    const int oh = s_offh[t], ow = s_offw[t];
                    const int h = h0 + oh, w = w0 + ow;
                    const bool in = t0 + tt < a.ntaps && (unsigned)h < (unsigned)a.H && (unsigned)w < (unsigned)a.W;
                    const unsigned off = base + (unsigned)((oh * a.W + ow) * C * (int)sizeof(T));
                    xv[tt] = __builtin_bit_cast(Vec, __builtin_amdgcn_raw_buffer_load_b128(xrsrc, in ? off : ~0u, 0, 0));
                }
                float df[VEC];
#pragma unroll
                for (int e = 0; e < VEC; ++e) df[e] = (float)dv[e];
#pragma unroll
                for (int tt = 0; tt < TC; ++tt) {
                    float xf[VEC];
#pragma unroll
                    for (int e = 0; e < VEC; ++e) xf[e] = (float)xv[tt][e];
#pragma unroll
                    for (int e = 0; e < VEC; ++e)
#pragma unroll
                        for (int cl = 0; cl < CG; ++cl) acc[tt][e][cl] += df[e] * xf[(e / CG) * CG + cl];
                }
            }
        // combine the pixel lanes, one (tap, channel of the group) at a time, in a fixed order
#pragma unroll
        for (int tt = 0; tt < TC; ++tt) {
            const int t = t0 + tt;
            if (t >= a.ntaps) break;    // uniform over the block
#pragma unroll
            for (int cl = 0; cl < CG; ++cl) {
                if (active)
#pragma unroll
                    for (int e = 0; e < VEC; ++e) red[pl * (cvb * VEC) + cvl * VEC + e] = acc[tt][e][cl];
                __syncthreads();
                if (tid < cvb * VEC) {
                    float s = 0.f;
                    for (int r = 0; r < PL; ++r) s += red[r * (cvb * VEC) + tid];
                    const int c = blockIdx.x * DW_CVB * VEC + tid;
                    part[((long)c * a.ntaps + t) * CG + cl] = s;
                }
                __syncthreads();
            }
        }
    }
}

bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace

bool depthwise_applicable(int dtype, const IgemmArgs &a)
{
    const int vec = dtype == NSK_BF16 ? 8 : 4, cg = a.Cs;
    // (eight channels per group fill a bf16 channel vector exactly; an fp32 vector holds four)
    if (!(a.groups > 1 && (cg == 1 || cg == 2 || cg == 4 || (cg == 8 && dtype == NSK_BF16)) && a.Ngemm == cg)) return false;
    const int C = a.groups * cg;
    const long words = dtype == NSK_BF16 ? (cg + 1) / 2 : cg;
    return a.src_ld == C && a.Co == C && C % vec == 0 && (long)a.ntaps * C * words * 4 <= DW_LDS_MAX && a.ntaps >= 1 &&
           !a.stats && aligned16(a.src) && aligned16(a.out);
}

template <typename T, int CG> int launch_depthwise_typed(const IgemmArgs &a, hipStream_t stream)
{
    constexpr int VEC = DTraits<T>::VEC;
    const int C = a.groups * CG;
    RowPlan rp{};
    ColPlan cp{};
    // the variables are test hooks; the column arrangement is preferred (contiguous loads)
    const bool cols = !hooks().depthwise_no_cols && !hooks().depthwise_no_rows && col_plan(a, &cp);
    const bool rows = !cols && !hooks().depthwise_no_rows && row_plan(a, &rp);
    const int S = rows ? a.ntaps / rp.R : 0, R = cols ? a.ntaps / cp.S : 0;
    const long threads = cols   ? (long)a.Nimg * ((a.Mi + DW_PIX - 1) / DW_PIX) * a.Mj * (C / VEC)
                         : rows ? (long)a.Nimg * a.Mi * ((a.Mj + DW_PIX - 1) / DW_PIX) * (C / VEC)
                                : ((long)a.M + DW_PIX - 1) / DW_PIX * (C / VEC);
    const long runs = (threads + 255) / 256;
    // enough blocks to fill the chip several times over, each with as many runs as that leaves (at most 8)
    int iters = (int)(runs / 2048);
    iters = iters < 1 ? 1 : (iters > 8 ? 8 : iters);
    const unsigned blocks = (unsigned)((runs + iters - 1) / iters);
    const size_t lds = (size_t)a.ntaps * C * lds_words<T, CG>() * sizeof(unsigned);
    if (R == 3)
        hipLaunchKernelGGL((depthwise_col_kernel<T, CG, 3>), dim3(blocks), dim3(256), lds, stream, a, cp, iters);
    else if (R == 5)
        hipLaunchKernelGGL((depthwise_col_kernel<T, CG, 5>), dim3(blocks), dim3(256), lds, stream, a, cp, iters);
    else if (R == 7)
        hipLaunchKernelGGL((depthwise_col_kernel<T, CG, 7>), dim3(blocks), dim3(256), lds, stream, a, cp, iters);
    else if (S == 3)
        hipLaunchKernelGGL((depthwise_row_kernel<T, CG, 3>), dim3(blocks), dim3(256), lds, stream, a, rp, iters);
    else if (S == 5)
        hipLaunchKernelGGL((depthwise_row_kernel<T, CG, 5>), dim3(blocks), dim3(256), lds, stream, a, rp, iters);
    else if (S == 7)
        hipLaunchKernelGGL((depthwise_row_kernel<T, CG, 7>), dim3(blocks), dim3(256), lds, stream, a, rp, iters);
    else
        hipLaunchKernelGGL((depthwise_kernel<T, CG>), dim3(blocks), dim3(256), lds, stream, a, iters);
    return check_launch();
}

int launch_depthwise(int dtype, const IgemmArgs &a, hipStream_t stream)
{
    if (dtype == NSK_BF16) {
        if (a.Cs == 1) return launch_depthwise_typed<bf16_t, 1>(a, stream);
        if (a.Cs == 2) return launch_depthwise_typed<bf16_t, 2>(a, stream);
        if (a.Cs == 8) return launch_depthwise_typed<bf16_t, 8>(a, stream);
        return launch_depthwise_typed<bf16_t, 4>(a, stream);
    }
    if (a.Cs == 1) return launch_depthwise_typed<float, 1>(a, stream);
    if (a.Cs == 2) return launch_depthwise_typed<float, 2>(a, stream);
    return launch_depthwise_typed<float, 4>(a, stream);
}

bool depthwise_wgrad_applicable(int dtype, const WgradArgs &a)
{
    const int vec = dtype == NSK_BF16 ? 8 : 4, cg = a.C;
    if (!(a.groups > 1 && (cg == 1 || cg == 2 || cg == 4 || (cg == 8 && dtype == NSK_BF16)) && a.K == cg)) return false;
    const int C = a.groups * cg;
    return a.ldx == C && a.ldy == C && C % vec == 0 && a.splits >= 1 && a.splits <= 65535 && aligned16(a.x) &&
           aligned16(a.dy);
}

template <typename T, int CG> int launch_depthwise_wgrad_typed(const WgradArgs &a, hipStream_t stream)
{
    dim3 grid(ceil_div(a.groups * CG / DTraits<T>::VEC, DW_CVB), a.splits);
    hipLaunchKernelGGL((depthwise_wgrad_kernel<T, CG>), grid, dim3(256), 0, stream, a);
    return check_launch();
}

int launch_depthwise_wgrad(int dtype, const WgradArgs &a, hipStream_t stream)
{
    if (dtype == NSK_BF16) {
        if (a.C == 1) return launch_depthwise_wgrad_typed<bf16_t, 1>(a, stream);
        if (a.C == 2) return launch_depthwise_wgrad_typed<bf16_t, 2>(a, stream);
        if (a.C == 8) return launch_depthwise_wgrad_typed<bf16_t, 8>(a, stream);
        return launch_depthwise_wgrad_typed<bf16_t, 4>(a, stream);
    }
    if (a.C == 1) return launch_depthwise_wgrad_typed<float, 1>(a, stream);
    if (a.C == 2) return launch_depthwise_wgrad_typed<float, 2>(a, stream);
    return launch_depthwise_wgrad_typed<float, 4>(a, stream);
}

}  // namespace nsk

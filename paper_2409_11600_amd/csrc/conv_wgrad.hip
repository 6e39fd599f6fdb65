// Backward-weight convolution: dw[k][tap][c] = sum over output pixels l = (img,p,q) of
// dy[l][k] * x[pixel(l) shifted by tap][c]  -- the weight gradient the paper accumulates into
// its gradient cache (section "Caching and Pooling").
//
// GEMM view: rows = output channels k, columns = (tap, input channel), reduction over the
// N*P*Q output pixels.  The output is tiny and the reduction is long, so the reduction is split
// across blocks (blockIdx.z) into float partials that a second kernel adds in a fixed order:
// results are bitwise reproducible, no floating-point atomics.
//
// Block tile: 64 rows x (64*FN) columns, four wavefronts as 2 x 2, each owning a 32 x (32*FN) strip
// of 32x32 MFMA accumulators.  FN = 3 makes a column tile exactly one filter row of a 3x3 filter with
// 64 channels, so x is re-read three times (not nine) across column tiles and every barrier is
// followed by three times as many MFMAs.
//
// Both operands are stored channel-contiguous, i.e. with the REDUCTION index as the slow one.
//  - fp32 (mfma 32x32x2, one k per lane): the tile is kept in LDS as [pixel][channel], exactly
//    as loaded, and a fragment is one conflict-free 4-byte read per lane.
//  - bf16 (mfma 32x32x16, 8 consecutive k per lane): the tile is transposed on the way into LDS
//    ([channel][pixel]) so that a fragment is one 16-byte read.
#include <stdlib.h>

#include "nsk_internal.h"

namespace nsk {
namespace {

constexpr int WBM = 64;

template <typename T> struct WTraits;
template <> struct WTraits<float> {
    static constexpr int VEC = 4, BK = 16;
    typedef f32x4 Vec;
};
template <> struct WTraits<bf16_t> {
    static constexpr int VEC = 8, BK = 32;
    typedef bf16x8 Vec;
};

template <typename T, int FN, bool VECLOAD>
__global__ __launch_bounds__(256) void wgrad_kernel(const WgradArgs a)
{
    typedef WTraits<T> TR;
    typedef typename TR::Vec Vec;
    constexpr int VEC = TR::VEC, BK = TR::BK;
    constexpr bool F32 = sizeof(T) == 4;
    constexpr int WBN = 64 * FN;
    // fp32: [BK][cols+4] (pixel-major) ; bf16: [cols][BK+8] (channel-major, pixel contiguous)
    constexpr int LDA = F32 ? (WBM + 4) : (BK + 8);
    constexpr int LDB = F32 ? (WBN + 4) : (BK + 8);
    constexpr int TILE_A = F32 ? BK * LDA : WBM * LDA;
    constexpr int TILE_B = F32 ? BK * LDB : WBN * LDB;
    constexpr int VPR_A = WBM / VEC;       // vectors per pixel row of the dy tile (BK * VPR_A = 256)
    constexpr int VPR_B = WBN / VEC;
    constexpr int B_LOADS = FN;            // vectors of the x tile per thread
    __shared__ __attribute__((aligned(16))) T As[2][TILE_A];
    __shared__ __attribute__((aligned(16))) T Bs[2][TILE_B];
    __shared__ short s_offh[kMaxTaps], s_offw[kMaxTaps];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int frow = lane & 31, fk = lane >> 5;
    // grouped convolution: blockIdx.z = group * splits + split (one group for a plain launch)
    const int grp = blockIdx.z / a.splits, split = blockIdx.z - grp * a.splits;
    const int n0 = blockIdx.x * WBN, k0 = blockIdx.y * WBM;
    const int ldx = a.ldx, ldy = a.ldy;
    const int NT = a.ntaps * a.C;
    if (tid < kMaxTaps) {
        s_offh[tid] = a.off_h[tid];
        s_offw[tid] = a.off_w[tid];
    }
    __syncthreads();

    const T *__restrict__ x = (const T *)a.x + (long)grp * a.C;     // the group's channel runs
    const T *__restrict__ dy = (const T *)a.dy + (long)grp * a.K;

    // thread -> (pixel row of the tile, vector of channels); bf16 keeps lanes along the pixel index so
    // the transposing 2-byte LDS writes of a wavefront fall into consecutive addresses.
    const int la = F32 ? tid / VPR_A : tid % BK;
    const int va = F32 ? tid % VPR_A : tid / BK;
    int lb[B_LOADS], vb[B_LOADS];
#pragma unroll
    for (int u = 0; u < B_LOADS; ++u) {
        const int idx = tid + 256 * u;
        lb[u] = F32 ? idx / VPR_B : idx % BK;
        vb[u] = F32 ? idx % VPR_B : idx / BK;
    }

    const int l_begin = split * a.rows_per_split;
    const int l_end = min(a.L, l_begin + a.rows_per_split);
    const int nk = (l_end - l_begin + BK - 1) / BK;

    // column (tap, channel) of this thread's x vectors: fixed for the whole loop
    int b_c[B_LOADS], b_oh[B_LOADS], b_ow[B_LOADS];
    bool b_ok[B_LOADS];
#pragma unroll
    for (int u = 0; u < B_LOADS; ++u) {
        const int n = n0 + vb[u] * VEC;
        b_ok[u] = VECLOAD && n < NT;
        b_c[u] = b_oh[u] = b_ow[u] = 0;
        if (b_ok[u]) {
            const int tap = n / a.C;
            b_c[u] = n - tap * a.C;
            b_oh[u] = s_offh[tap];
            b_ow[u] = s_offw[tap];
        }
    }
    const int kA = k0 + va * VEC;

    Vec ra, rb[B_LOADS];
    auto zero = [](Vec &v) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] = 0;
    };
    auto decode = [&](int l, int &img, int &p, int &q) {
        const int pq = a.P * a.Q;
        img = l / pq;
        const int rem = l - img * pq;
        p = rem / a.Q;
        q = rem - p * a.Q;
    };
    auto load_tile = [&](int kt) {
        const int base = l_begin + kt * BK;
        zero(ra);
        {
            const int l = base + la;
            if (l < l_end) {
                if (VECLOAD) {
                    if (kA < a.K) ra = *(const Vec *)(dy + (long)l * ldy + kA);
                } else {
#pragma unroll
                    for (int e = 0; e < VEC; ++e)
                        if (kA + e < a.K) ra[e] = dy[(long)l * ldy + kA + e];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < B_LOADS; ++u) {
            zero(rb[u]);
            const int l = base + lb[u];
            if (l >= l_end) continue;
            int img, p, q;
            decode(l, img, p, q);
            if (VECLOAD) {
                if (b_ok[u]) {
                    const int h = p * a.sh - a.ph + b_oh[u], w = q * a.sw - a.pw + b_ow[u];
                    if ((unsigned)h < (unsigned)a.H && (unsigned)w < (unsigned)a.W)
                        rb[u] = *(const Vec *)(x + (((long)img * a.H + h) * a.W + w) * ldx + b_c[u]);
                }
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const int n = n0 + vb[u] * VEC + e;
                    if (n < NT) {
                        const int tap = n / a.C;
                        const int c = n - tap * a.C;
                        const int h = p * a.sh - a.ph + s_offh[tap], w = q * a.sw - a.pw + s_offw[tap];
                        if ((unsigned)h < (unsigned)a.H && (unsigned)w < (unsigned)a.W)
                            rb[u][e] = x[(((long)img * a.H + h) * a.W + w) * ldx + c];
                    }
                }
            }
        }
    };
    auto store_tile = [&](int buf) {
        if constexpr (F32) {
            *(Vec *)&As[buf][la * LDA + va * VEC] = ra;
#pragma unroll
            for (int u = 0; u < B_LOADS; ++u) *(Vec *)&Bs[buf][lb[u] * LDB + vb[u] * VEC] = rb[u];
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) As[buf][(va * VEC + e) * LDA + la] = ra[e];
#pragma unroll
            for (int u = 0; u < B_LOADS; ++u)
#pragma unroll
                for (int e = 0; e < VEC; ++e) Bs[buf][(vb[u] * VEC + e) * LDB + lb[u]] = rb[u][e];
        }
    };

    f32x16 acc[FN];
#pragma unroll
    for (int ni = 0; ni < FN; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[ni][v] = 0.f;

    if (nk > 0) {
        load_tile(0);
        store_tile(0);
    }
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_tile(kt + 1);
        if constexpr (F32) {
#pragma unroll
            for (int t = 0; t < BK / 2; ++t) {
                const float av = As[buf][(2 * t + fk) * LDA + wm * 32 + frow];
#pragma unroll
                for (int ni = 0; ni < FN; ++ni) {
                    const float bv = Bs[buf][(2 * t + fk) * LDB + (wn * FN + ni) * 32 + frow];
                    acc[ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[ni], 0, 0, 0);
                }
            }
        } else {
#pragma unroll
            for (int ks = 0; ks < BK; ks += 16) {
                const Vec av = *(const Vec *)&As[buf][(wm * 32 + frow) * LDA + ks + 8 * fk];
#pragma unroll
                for (int ni = 0; ni < FN; ++ni) {
                    const Vec bv = *(const Vec *)&Bs[buf][((wn * FN + ni) * 32 + frow) * LDB + ks + 8 * fk];
                    acc[ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc[ni], 0, 0, 0);
                }
            }
        }
        if (kt + 1 < nk) store_tile(buf ^ 1);
        __syncthreads();
    }

    float *__restrict__ part = a.part + ((long)split * a.groups + grp) * a.K * NT;
#pragma unroll
    for (int ni = 0; ni < FN; ++ni) {
        const int col = n0 + (wn * FN + ni) * 32 + frow;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int k = k0 + wm * 32 + 8 * (v >> 2) + 4 * fk + (v & 3);
            if (k < a.K && col < NT) part[(long)k * NT + col] = acc[ni][v];
        }
    }
}

// dw[...] (=|+=) sum over splits of part[split][i], splits taken in four interleaved groups that
// are combined in a fixed order (reproducible).  One block covers 64 consecutive outputs.
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float *__restrict__ part, float *__restrict__ dw,
                                                            int splits, int K, int ntaps, int C, long sk, long st,
                                                            long sc, int accumulate)
{
    __shared__ float red[4][64];
    const long total = (long)K * ntaps * C;
    const int g = threadIdx.x >> 6;
    const long i = (long)blockIdx.x * 64 + (threadIdx.x & 63);
    float s = 0.f;
    if (i < total)
#pragma unroll 8
        for (int sp = g; sp < splits; sp += 4) s += part[(long)sp * total + i];
    red[g][threadIdx.x & 63] = s;
    __syncthreads();
    if (g != 0 || i >= total) return;
    s = (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
    const int c = (int)(i % C);
    const long r = i / C;
    const int t = (int)(r % ntaps);
    const long k = r / ntaps;
    float *o = dw + k * sk + t * st + c * sc;
    *o = accumulate ? *o + s : s;
}

// The same sums in the same order for outputs that lie in dw as they lie in a partial sum (NHWC, one group): a lane takes
// V consecutive outputs with one 8- or 16-byte load per split, so a wavefront's load is 512 or 1024 contiguous bytes.
template <int V>
__global__ __launch_bounds__(256) void wgrad_reduce_vec_kernel(const float *__restrict__ part, float *__restrict__ dw,
                                                                int splits, long total, int accumulate)
{
    typedef float fv __attribute__((ext_vector_type(V)));
    __shared__ fv red[4][64];
    const int g = threadIdx.x >> 6, l = threadIdx.x & 63;
    const long i = ((long)blockIdx.x * 64 + l) * V;      // total % V == 0: a vector is inside or outside as a whole
    fv s;
#pragma unroll
    for (int e = 0; e < V; ++e) s[e] = 0.f;
    if (i < total)
#pragma unroll 8
        for (int sp = g; sp < splits; sp += 4) s += *(const fv *)(part + (long)sp * total + i);
    red[g][l] = s;
    __syncthreads();
    if (g != 0 || i >= total) return;
    s = (red[0][l] + red[1][l]) + (red[2][l] + red[3][l]);
    fv *o = (fv *)(dw + i);
    *o = accumulate ? *o + s : s;
}

// The same for small outputs with many splits (the 16- and 32-channel layers and the 3-channel stem of the CIFAR-sized
// network: a few thousand outputs, hundreds of splits): 16 interleaved groups of splits instead of four, so that a lane's
// chain of dependent loads is a quarter as long.  One block covers 16 consecutive outputs; fixed order as above.
__global__ __launch_bounds__(256) void wgrad_reduce16_kernel(const float *__restrict__ part, float *__restrict__ dw,
                                                              int splits, int K, int ntaps, int C, long sk, long st,
                                                              long sc, int accumulate)
{
    __shared__ float red[16][16];
    const long total = (long)K * ntaps * C;
    const int g = threadIdx.x >> 4, j = threadIdx.x & 15;
    const long i = (long)blockIdx.x * 16 + j;
    float s = 0.f;
    if (i < total)
#pragma unroll 4
        for (int sp = g; sp < splits; sp += 16) s += part[(long)sp * total + i];
    red[g][j] = s;
    __syncthreads();
    if (g != 0 || i >= total) return;
    float r = 0.f;
#pragma unroll
    for (int q = 0; q < 16; q += 4) r += (red[q][j] + red[q + 1][j]) + (red[q + 2][j] + red[q + 3][j]);
    const int c = (int)(i % C);
    const long rr = i / C;
    const int t = (int)(rr % ntaps);
    const long k = rr / ntaps;
    float *o = dw + k * sk + t * st + c * sc;
    *o = accumulate ? *o + r : r;
}

int column_frags(int ntapsC) { return ntapsC % 192 == 0 ? 3 : 1; }

}  // namespace

int wgrad_rows_per_split(int dtype, int L, int K, int ntapsC, int *splits)
{
    const int BK = dtype == NSK_BF16 ? WTraits<bf16_t>::BK : WTraits<float>::BK;
    const long tiles = (long)ceil_div(K, WBM) * ceil_div(ntapsC, 64 * column_frags(ntapsC));
    long want = (768 + tiles - 1) / tiles;  // about three blocks per CU
    const long most = (L + 4 * BK - 1) / (4 * BK);
    if (want > most) want = most;
    if (want < 1) want = 1;
    int rows = (int)((L + want - 1) / want);
    rows = ceil_div(rows, BK) * BK;
    *splits = ceil_div(L, rows);
    return rows;
}

template <typename T> int launch_wgrad_typed(const WgradArgs &a, bool vec, hipStream_t stream)
{
    const int NT = a.ntaps * a.C;
    const int fn = column_frags(NT);
    dim3 grid(ceil_div(NT, 64 * fn), ceil_div(a.K, WBM), a.splits * a.groups);
    if (fn == 3) {
        if (vec)
            hipLaunchKernelGGL((wgrad_kernel<T, 3, true>), grid, dim3(256), 0, stream, a);
        else
            hipLaunchKernelGGL((wgrad_kernel<T, 3, false>), grid, dim3(256), 0, stream, a);
    } else {
        if (vec)
            hipLaunchKernelGGL((wgrad_kernel<T, 1, true>), grid, dim3(256), 0, stream, a);
        else
            hipLaunchKernelGGL((wgrad_kernel<T, 1, false>), grid, dim3(256), 0, stream, a);
    }
    return check_launch();
}

int launch_wgrad(int dtype, const WgradArgs &a0, hipStream_t stream)
{
    WgradArgs a = a0;
    if (a.groups > 1) {
        if (a.ldx != a.groups * a.C || a.ldy != a.groups * a.K || (long)a.groups * a.splits > 65535) return NSK_ERR_BAD_DESC;
    } else {
        a.groups = 1;
        a.ldx = a.C;
        a.ldy = a.K;
    }
    if (tiny_wgrad_applicable(dtype, a)) return launch_tiny_wgrad(dtype, a, stream);
    if (!hooks().no_depthwise && depthwise_wgrad_applicable(dtype, a)) return launch_depthwise_wgrad(dtype, a, stream);
    const int VEC = dtype == NSK_BF16 ? 8 : 4;
    // (with C and K multiples of VEC every group's channel runs start on 16-byte boundaries too)
    const bool vec = a.C % VEC == 0 && a.K % VEC == 0 && (uintptr_t)a.x % 16 == 0 && (uintptr_t)a.dy % 16 == 0;
    if (dtype == NSK_BF16) return launch_wgrad_typed<bf16_t>(a, vec, stream);
    return launch_wgrad_typed<float>(a, vec, stream);
}

int launch_wgrad_reduce(const float *part, float *dw, int splits, int K, int ntaps, int C, long sk,
                        long st, long sc, int accumulate, hipStream_t stream)
{
    const long total = (long)K * ntaps * C;
    // dw in the order of the partial sums: vector loads (bitwise the same sums); enough blocks to cover the chip
    const bool flat = sc == 1 && st == (long)C && sk == (long)ntaps * C && !hooks().reduce4 &&
                      (((uintptr_t)part | (uintptr_t)dw) & 15) == 0;
    if (flat && total % 4 == 0 && total >= 4 * 64 * 512) {
        hipLaunchKernelGGL(wgrad_reduce_vec_kernel<4>, dim3((unsigned)((total / 4 + 63) / 64)), dim3(256), 0, stream, part, dw, splits, total, accumulate);
        return check_launch();
    }
    if (flat && total % 2 == 0 && total >= 2 * 64 * 256) {
        hipLaunchKernelGGL(wgrad_reduce_vec_kernel<2>, dim3((unsigned)((total / 2 + 63) / 64)), dim3(256), 0, stream, part, dw, splits, total, accumulate);
        return check_launch();
    }
    if (total <= 16384 && splits >= 64 && !hooks().reduce4)   // (the variable is an A/B hook)
        hipLaunchKernelGGL(wgrad_reduce16_kernel, dim3((unsigned)((total + 15) / 16)), dim3(256), 0, stream, part, dw,
                           splits, K, ntaps, C, sk, st, sc, accumulate);
    else
        hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)((total + 63) / 64)), dim3(256), 0, stream, part, dw,
                           splits, K, ntaps, C, sk, st, sc, accumulate);
    return check_launch();
}

}  // namespace nsk

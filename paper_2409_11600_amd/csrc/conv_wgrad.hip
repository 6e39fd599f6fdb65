// Backward-weight convolution: dw[k][tap][c] = sum over output pixels l = (img,p,q) of
// dy[l][k] * x[pixel(l) shifted by tap][c]  -- the weight gradient the paper accumulates into
// its gradient cache (section "Caching and Pooling").
//
// GEMM view: rows = output channels k, columns = (tap, input channel), reduction over the
// N*P*Q output pixels.  The output is tiny and the reduction is long, so the reduction is split
// across blocks (blockIdx.z) into float partials that a second kernel adds in a fixed order:
// results are bitwise reproducible, no floating-point atomics.
//
// Both operands are stored channel-contiguous, i.e. with the REDUCTION index as the slow one.
//  - fp32 (mfma 32x32x2, one k per lane): the tile is kept in LDS as [pixel][channel], exactly
//    as loaded, and a fragment is one conflict-free 4-byte read per lane.
//  - bf16 (mfma 32x32x16, 8 consecutive k per lane): the tile is transposed on the way into LDS
//    ([channel][pixel]) so that a fragment is one 16-byte read.
#include "nsk_internal.h"

namespace nsk {
namespace {

constexpr int WBM = 64, WBN = 64;

template <typename T> struct WTraits;
template <> struct WTraits<float> {
    static constexpr int VEC = 4, BK = 16;
    typedef f32x4 Vec;
};
template <> struct WTraits<bf16_t> {
    static constexpr int VEC = 8, BK = 32;
    typedef bf16x8 Vec;
};

template <typename T, bool VECLOAD>
__global__ __launch_bounds__(256) void wgrad_kernel(const WgradArgs a)
{
    typedef WTraits<T> TR;
    typedef typename TR::Vec Vec;
    constexpr int VEC = TR::VEC, BK = TR::BK;
    constexpr bool F32 = sizeof(T) == 4;
    // fp32: [BK][64+4] (pixel-major) ; bf16: [64][BK+8] (channel-major, pixel contiguous)
    constexpr int LD = F32 ? (64 + 4) : (BK + 8);
    constexpr int TILE = F32 ? BK * LD : 64 * LD;
    constexpr int VPR = 64 / VEC;          // vectors per pixel row of the tile
    __shared__ __attribute__((aligned(16))) T As[2][TILE];
    __shared__ __attribute__((aligned(16))) T Bs[2][TILE];
    __shared__ short s_offh[kMaxTaps], s_offw[kMaxTaps];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int frow = lane & 31, fk = lane >> 5;
    const int n0 = blockIdx.x * WBN, k0 = blockIdx.y * WBM, split = blockIdx.z;
    const int NT = a.ntaps * a.C;
    if (tid < kMaxTaps) {
        s_offh[tid] = a.off_h[tid];
        s_offw[tid] = a.off_w[tid];
    }
    __syncthreads();

    const T *__restrict__ x = (const T *)a.x;
    const T *__restrict__ dy = (const T *)a.dy;

    // thread -> (pixel row of the tile, vector of 64 channels); bf16 keeps lanes along the pixel
    // index so the transposing 2-byte LDS writes of a wavefront fall into consecutive addresses.
    const int l_loc = F32 ? tid / VPR : tid % BK;
    const int vv = F32 ? tid % VPR : tid / BK;

    const int l_begin = split * a.rows_per_split;
    const int l_end = min(a.L, l_begin + a.rows_per_split);
    const int nk = (l_end - l_begin + BK - 1) / BK;

    // column (tap, channel) of this thread's B vector: fixed for the whole loop
    const int nB = n0 + vv * VEC;
    int b_tap = 0, b_c = 0, b_oh = 0, b_ow = 0;
    bool b_col_ok = false;
    if (VECLOAD) {
        b_col_ok = nB < NT;
        if (b_col_ok) {
            b_tap = nB / a.C;
            b_c = nB - b_tap * a.C;
            b_oh = s_offh[b_tap];
            b_ow = s_offw[b_tap];
        }
    }
    const int kA = k0 + vv * VEC;

    Vec ra, rb;
    auto zero = [](Vec &v) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] = 0;
    };
    auto load_tile = [&](int kt) {
        const int l = l_begin + kt * BK + l_loc;
        zero(ra);
        zero(rb);
        if (l >= l_end) return;
        const int pq = a.P * a.Q;
        const int img = l / pq;
        const int rem = l - img * pq;
        const int p = rem / a.Q;
        const int q = rem - p * a.Q;
        if (VECLOAD) {
            if (kA < a.K) ra = *(const Vec *)(dy + (long)l * a.K + kA);
            if (b_col_ok) {
                const int h = p * a.sh - a.ph + b_oh, w = q * a.sw - a.pw + b_ow;
                if ((unsigned)h < (unsigned)a.H && (unsigned)w < (unsigned)a.W)
                    rb = *(const Vec *)(x + (((long)img * a.H + h) * a.W + w) * a.C + b_c);
            }
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                if (kA + e < a.K) ra[e] = dy[(long)l * a.K + kA + e];
                const int n = nB + e;
                if (n < NT) {
                    const int tap = n / a.C;
                    const int c = n - tap * a.C;
                    const int h = p * a.sh - a.ph + s_offh[tap], w = q * a.sw - a.pw + s_offw[tap];
                    if ((unsigned)h < (unsigned)a.H && (unsigned)w < (unsigned)a.W)
                        rb[e] = x[(((long)img * a.H + h) * a.W + w) * a.C + c];
                }
            }
        }
    };
    auto store_tile = [&](int buf) {
        if constexpr (F32) {
            *(Vec *)&As[buf][l_loc * LD + vv * VEC] = ra;
            *(Vec *)&Bs[buf][l_loc * LD + vv * VEC] = rb;
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                As[buf][(vv * VEC + e) * LD + l_loc] = ra[e];
                Bs[buf][(vv * VEC + e) * LD + l_loc] = rb[e];
            }
        }
    };

    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;

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
                const float av = As[buf][(2 * t + fk) * LD + wm * 32 + frow];
                const float bv = Bs[buf][(2 * t + fk) * LD + wn * 32 + frow];
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc, 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int ks = 0; ks < BK; ks += 16) {
                const Vec av = *(const Vec *)&As[buf][(wm * 32 + frow) * LD + ks + 8 * fk];
                const Vec bv = *(const Vec *)&Bs[buf][(wn * 32 + frow) * LD + ks + 8 * fk];
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc, 0, 0, 0);
            }
        }
        if (kt + 1 < nk) store_tile(buf ^ 1);
        __syncthreads();
    }

    float *__restrict__ part = a.part + (long)split * a.K * NT;
    const int col = n0 + wn * 32 + frow;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int k = k0 + wm * 32 + 8 * (v >> 2) + 4 * fk + (v & 3);
        if (k < a.K && col < NT) part[(long)k * NT + col] = acc[v];
    }
}

__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float *__restrict__ part, float *__restrict__ dw,
                                                            int splits, int K, int ntaps, int C, long sk, long st,
                                                            long sc, int accumulate)
{
    const long total = (long)K * ntaps * C;
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    float s = 0.f;
    for (int sp = 0; sp < splits; ++sp) s += part[(long)sp * total + i];
    const int c = (int)(i % C);
    const long r = i / C;
    const int t = (int)(r % ntaps);
    const long k = r / ntaps;
    float *o = dw + k * sk + t * st + c * sc;
    *o = accumulate ? *o + s : s;
}

}  // namespace

int wgrad_rows_per_split(int dtype, int L, int K, int ntapsC, int *splits)
{
    const int BK = dtype == NSK_BF16 ? WTraits<bf16_t>::BK : WTraits<float>::BK;
    const long tiles = (long)ceil_div(K, WBM) * ceil_div(ntapsC, WBN);
    long want = (1024 + tiles - 1) / tiles;
    const long most = (L + 4 * BK - 1) / (4 * BK);
    if (want > most) want = most;
    if (want < 1) want = 1;
    int rows = (int)((L + want - 1) / want);
    rows = ceil_div(rows, BK) * BK;
    *splits = ceil_div(L, rows);
    return rows;
}

int launch_wgrad(int dtype, const WgradArgs &a, hipStream_t stream)
{
    const int NT = a.ntaps * a.C;
    dim3 grid(ceil_div(NT, WBN), ceil_div(a.K, WBM), a.splits);
    const int VEC = dtype == NSK_BF16 ? 8 : 4;
    const bool vec = a.C % VEC == 0 && a.K % VEC == 0 && (uintptr_t)a.x % 16 == 0 && (uintptr_t)a.dy % 16 == 0;
    if (dtype == NSK_BF16) {
        if (vec)
            hipLaunchKernelGGL((wgrad_kernel<bf16_t, true>), grid, dim3(256), 0, stream, a);
        else
            hipLaunchKernelGGL((wgrad_kernel<bf16_t, false>), grid, dim3(256), 0, stream, a);
    } else {
        if (vec)
            hipLaunchKernelGGL((wgrad_kernel<float, true>), grid, dim3(256), 0, stream, a);
        else
            hipLaunchKernelGGL((wgrad_kernel<float, false>), grid, dim3(256), 0, stream, a);
    }
    return check_launch();
}

int launch_wgrad_reduce(const float *part, float *dw, int splits, int K, int ntaps, int C, long sk,
                        long st, long sc, int accumulate, hipStream_t stream)
{
    const long total = (long)K * ntaps * C;
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, part, dw,
                       splits, K, ntaps, C, sk, st, sc, accumulate);
    return check_launch();
}

}  // namespace nsk

// Convolution layers with at most four channels on one side and 8..64 on the other: the stride-1 image stem of the
// small-image residual network the paper trains on CIFAR-10 (3 -> 16 channels, section "Experiments and Discussion").
// A 3-channel pixel is 6 bytes, so the implicit-GEMM kernels can only gather it element by element into tiles that
// are mostly padding (24 / 26 / 52 us for a layer whose tensors stream in 3 us).  There is next to no arithmetic
// here (432 multiply-adds per pixel), so the three passes are direct kernels on the vector ALUs, bound by memory:
//   * forward (few source channels): a lane owns one output pixel and all its NG output channels; the filter lies in
//     LDS as floats [tap][source channel][NG] and is read by broadcast;
//   * backward-data (few output channels): a lane owns one output pixel, loads the CS source channels of each tap's
//     pixel with 16-byte loads and multiplies them with the filter rows [tap][output channel][CS] from LDS;
//   * backward-weight: a lane owns two (tap, input channel) columns of dw for all K output channels; the 16 column
//     lanes of a pixel lane read the same dy vector (broadcast) and their own x elements; sixteen pixel lanes per
//     block are combined through LDS in a fixed order.  Partial sums in the layout of the generic split kernel.
// Forward and backward-data take the argument set of the implicit-GEMM kernels (taps as offsets around a base pixel,
// strided output grid), so stride classes, padding, dilation and `accumulate` come for free.
#include <stdlib.h>

#include "nsk_internal.h"

namespace nsk {
namespace {

constexpr int TINY_MAX_C = 4;        // channels on the narrow side
constexpr int TINY_LDS_MAX = 48 << 10;
constexpr int TINY_PIX = 2;         // output pixels per lane of the forward kernel

__device__ inline float tf(float v) { return v; }
__device__ inline float tf(bf16_t v) { return (float)v; }

typedef bf16_t bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
// acc += x . w over the two bf16 halves of a dword (both halves are terms of the same sum wherever this is used)
__device__ inline float dot2(unsigned x, unsigned w, float acc)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, x), __builtin_bit_cast(bf16x2, w), acc, false);
}

// ---------------------------------------------------------------- forward: Cs <= 4 source channels, NG output channels
template <typename T, int NG>
__global__ __launch_bounds__(256) void tiny_src_kernel(const IgemmArgs a)
{
    constexpr int VEC = 16 / (int)sizeof(T);
    typedef T Vec __attribute__((ext_vector_type(VEC)));
    extern __shared__ __attribute__((aligned(16))) float wL[];   // [ntaps * Cs][NG]
    __shared__ short s_offh[kMaxTaps], s_offw[kMaxTaps];
    const int tid = threadIdx.x, Cs = a.Cs, Ktot = a.Ktot;
    const T *__restrict__ src = (const T *)a.src;
    const T *__restrict__ wpk = (const T *)a.wpk;   // [NG][Ktot]
    T *__restrict__ out = (T *)a.out;
    for (int i = tid; i < Ktot * NG; i += 256) {
        const int n = i / Ktot, k = i - n * Ktot;
        wL[k * NG + n] = tf(wpk[i]);
    }
    if (tid < kMaxTaps) {
        s_offh[tid] = a.off_h[tid];
        s_offw[tid] = a.off_w[tid];
    }
    __syncthreads();
    // a lane owns TINY_PIX consecutive output pixels: a filter row read from LDS (a broadcast, but it still costs the LDS
    // pipe a full pass) serves all of them
    const long m0 = ((long)blockIdx.x * 256 + tid) * TINY_PIX;
    if (m0 >= a.M) return;
    const int per_img = a.Mi * a.Mj;
    int bh[TINY_PIX], bw[TINY_PIX];
    long src_img[TINY_PIX], out_off[TINY_PIX];
    bool live[TINY_PIX];
    float acc[TINY_PIX][NG];
#pragma unroll
    for (int u = 0; u < TINY_PIX; ++u) {
        live[u] = m0 + u < a.M;
        const int m = live[u] ? (int)(m0 + u) : 0;
        const int img = m / per_img;
        const int rem = m - img * per_img;
        const int i = rem / a.Mj;
        const int j = rem - i * a.Mj;
        bh[u] = i * a.mult_h + a.add_h;
        bw[u] = j * a.mult_w + a.add_w;
        src_img[u] = (long)img * a.Hs;
        out_off[u] = (((long)img * a.Ho + (i * a.osh + a.oa)) * a.Wo + (j * a.osw + a.ob)) * a.Co;
#pragma unroll
        for (int n = 0; n < NG; ++n) acc[u][n] = 0.f;
        if (a.accumulate && live[u]) {   // start from the old values: the sum is rounded to the storage type once
#pragma unroll
            for (int v = 0; v < NG / VEC; ++v) {
                const Vec old = *(const Vec *)(out + out_off[u] + v * VEC);
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[u][v * VEC + e] = tf(old[e]);
            }
        }
    }
    // Every load is unconditional (coordinates clamped into the image, the value masked afterwards), so the loads of
    // several taps are in flight together instead of one dependent load per branch.
#pragma unroll 3
    for (int t = 0; t < a.ntaps; ++t) {
        float xv[TINY_PIX][TINY_MAX_C];
#pragma unroll
        for (int u = 0; u < TINY_PIX; ++u) {
            const int h = bh[u] + s_offh[t], w = bw[u] + s_offw[t];
            const bool in = live[u] && (unsigned)h < (unsigned)a.Hs && (unsigned)w < (unsigned)a.Ws;
            const int hc = min(max(h, 0), a.Hs - 1), wc = min(max(w, 0), a.Ws - 1);
            const T *px = src + ((src_img[u] + hc) * a.Ws + wc) * Cs;
#pragma unroll
            for (int c = 0; c < TINY_MAX_C; ++c) {
                const float v = tf(px[min(c, Cs - 1)]);
                xv[u][c] = (in && c < Cs) ? v : 0.f;
            }
        }
#pragma unroll
        for (int c = 0; c < TINY_MAX_C; ++c) {
            if (c >= Cs) break;   // uniform
            const float *wr = wL + (t * Cs + c) * NG;
#pragma unroll
            for (int n = 0; n < NG; n += 4) {
                const f32x4 q = *(const f32x4 *)(wr + n);
#pragma unroll
                for (int u = 0; u < TINY_PIX; ++u) {
                    acc[u][n] += xv[u][c] * q[0];
                    acc[u][n + 1] += xv[u][c] * q[1];
                    acc[u][n + 2] += xv[u][c] * q[2];
                    acc[u][n + 3] += xv[u][c] * q[3];
                }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < TINY_PIX; ++u) {
        if (!live[u]) continue;
#pragma unroll
        for (int v = 0; v < NG / VEC; ++v) {
            Vec o;
#pragma unroll
            for (int e = 0; e < VEC; ++e) o[e] = (T)acc[u][v * VEC + e];
            *(Vec *)(out + out_off[u] + v * VEC) = o;
        }
    }
}

// ---------------------------------------------------------------- backward-data: CS source channels, Ngemm <= 4 outputs
template <typename T, int CS>
__global__ __launch_bounds__(256) void tiny_out_kernel(const IgemmArgs a)
{
    constexpr int VEC = 16 / (int)sizeof(T);
    typedef T Vec __attribute__((ext_vector_type(VEC)));
    // filter rows [ntaps][TINY_MAX_C][CS] (rows n >= Ngemm are zero): floats for fp32, the bf16 values themselves
    // (two per dword) for bf16, whose products are two-element dot products on the raw dwords
    constexpr bool BF = sizeof(T) == 2;
    constexpr int WROW = BF ? CS / 2 : CS;       // LDS words per filter row
    extern __shared__ __attribute__((aligned(16))) float wL[];
    __shared__ short s_offh[kMaxTaps], s_offw[kMaxTaps];
    const int tid = threadIdx.x, NO = a.Ngemm;
    const T *__restrict__ src = (const T *)a.src;
    const T *__restrict__ wpk = (const T *)a.wpk;   // [NO][ntaps][CS]
    T *__restrict__ out = (T *)a.out;
    for (int i = tid; i < a.ntaps * TINY_MAX_C * WROW; i += 256) {
        const int c = i % WROW, r = i / WROW;
        const int n = r % TINY_MAX_C, t = r / TINY_MAX_C;
        if constexpr (BF) {
            const unsigned short *q = (const unsigned short *)wpk + ((long)n * a.ntaps + t) * CS + 2 * c;
            ((unsigned *)wL)[i] = n < NO ? ((unsigned)q[0] | ((unsigned)q[1] << 16)) : 0u;
        } else {
            wL[i] = n < NO ? tf(wpk[((long)n * a.ntaps + t) * CS + c]) : 0.f;
        }
    }
    if (tid < kMaxTaps) {
        s_offh[tid] = a.off_h[tid];
        s_offw[tid] = a.off_w[tid];
    }
    __syncthreads();
    const long m_ = (long)blockIdx.x * 256 + tid;
    if (m_ >= a.M) return;
    const int m = (int)m_;
    const int per_img = a.Mi * a.Mj;
    const int img = m / per_img;
    const int rem = m - img * per_img;
    const int i = rem / a.Mj;
    const int j = rem - i * a.Mj;
    const int bh = i * a.mult_h + a.add_h, bw = j * a.mult_w + a.add_w;
    const long out_off = (((long)img * a.Ho + (i * a.osh + a.oa)) * a.Wo + (j * a.osw + a.ob)) * a.Co;
    float acc[TINY_MAX_C];
#pragma unroll
    for (int n = 0; n < TINY_MAX_C; ++n) acc[n] = (a.accumulate && n < NO) ? tf(out[out_off + n]) : 0.f;
    // unconditional loads (clamped coordinates, masked values): the loads of consecutive taps overlap
#pragma unroll 2
    for (int t = 0; t < a.ntaps; ++t) {
        const int h = bh + s_offh[t], w = bw + s_offw[t];
        const bool in = (unsigned)h < (unsigned)a.Hs && (unsigned)w < (unsigned)a.Ws;
        const int hc = min(max(h, 0), a.Hs - 1), wc = min(max(w, 0), a.Ws - 1);
        const T *px = src + (((long)img * a.Hs + hc) * a.Ws + wc) * CS;
        Vec xv[CS / VEC];
#pragma unroll
        for (int v = 0; v < CS / VEC; ++v) xv[v] = *(const Vec *)(px + v * VEC);
        const float *wr = wL + t * TINY_MAX_C * WROW;
        if constexpr (BF) {
#pragma unroll
            for (int v = 0; v < CS / VEC; ++v) {
                const u32x4 xd = in ? __builtin_bit_cast(u32x4, xv[v]) : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
                for (int n = 0; n < TINY_MAX_C; ++n) {
                    const u32x4 q = *(const u32x4 *)(wr + n * WROW + v * 4);
                    acc[n] = dot2(xd[0], q[0], acc[n]);
                    acc[n] = dot2(xd[1], q[1], acc[n]);
                    acc[n] = dot2(xd[2], q[2], acc[n]);
                    acc[n] = dot2(xd[3], q[3], acc[n]);
                }
            }
        } else
#pragma unroll
        for (int v = 0; v < CS / VEC; ++v)
#pragma unroll
            for (int e = 0; e < VEC; e += 4) {
                const float x0 = in ? tf(xv[v][e]) : 0.f, x1 = in ? tf(xv[v][e + 1]) : 0.f,
                            x2 = in ? tf(xv[v][e + 2]) : 0.f, x3 = in ? tf(xv[v][e + 3]) : 0.f;
#pragma unroll
                for (int n = 0; n < TINY_MAX_C; ++n) {
                    const f32x4 q = *(const f32x4 *)(wr + n * CS + v * VEC + e);
                    acc[n] += x0 * q[0] + x1 * q[1] + x2 * q[2] + x3 * q[3];
                }
            }
    }
#pragma unroll
    for (int n = 0; n < TINY_MAX_C; ++n)
        if (n < NO) out[out_off + n] = (T)acc[n];
}

// ---------------------------------------------------------------- backward-weight: C <= 4 input channels, KT output channels
template <typename T, int KT>
__global__ __launch_bounds__(256) void tiny_wgrad_kernel(const WgradArgs a)
{
    constexpr int VEC = 16 / (int)sizeof(T);
    typedef T Vec __attribute__((ext_vector_type(VEC)));
    // A block covers COLS = 32 columns (tap, channel) of dw with 16 column lanes of two columns each (the conversion of
    // the K dy values is then shared by two columns' multiply-adds) and PL = 16 pixel lanes.
    constexpr int COLS = 32, CL = COLS / 2, PL = 256 / CL;
    __shared__ float red[PL * 16 * COLS];
    __shared__ short s_offh[kMaxTaps], s_offw[kMaxTaps];
    const int tid = threadIdx.x;
    const int NT = a.ntaps * a.C;
    const int lc = tid % CL, pl = tid / CL;
    const int split = blockIdx.y;
    const T *__restrict__ x = (const T *)a.x;
    const T *__restrict__ dy = (const T *)a.dy;
    if (tid < kMaxTaps) {
        s_offh[tid] = a.off_h[tid];
        s_offw[tid] = a.off_w[tid];
    }
    __syncthreads();
    bool live[2];
    int cc[2], oh[2], ow[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int col = blockIdx.x * COLS + 2 * lc + j;
        live[j] = col < NT;
        const int tap = live[j] ? col / a.C : 0;
        cc[j] = live[j] ? col - tap * a.C : 0;
        oh[j] = s_offh[tap];
        ow[j] = s_offw[tap];
    }
    const int l_begin = split * a.rows_per_split;
    const int l_end = min(a.L, l_begin + a.rows_per_split);
    const int pq = a.P * a.Q;
    float acc[2][KT];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int k = 0; k < KT; ++k) acc[j][k] = 0.f;
    // (img, p, q) of the lane's pixel: decoded once, then stepped (a division per pixel would cost more than its FMAs)
    int img, p, q;
    {
        const int l0 = min(l_begin + pl, a.L - 1);
        img = l0 / pq;
        const int rem = l0 - img * pq;
        p = rem / a.Q;
        q = rem - p * a.Q;
    }
#pragma unroll 2
    for (int l = l_begin + pl; l < l_end; l += PL) {
        float xv[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int h = p * a.sh - a.ph + oh[j], w = q * a.sw - a.pw + ow[j];
            const bool in = live[j] && (unsigned)h < (unsigned)a.H && (unsigned)w < (unsigned)a.W;
            const int hc = min(max(h, 0), a.H - 1), wc = min(max(w, 0), a.W - 1);   // unconditional load, masked value
            const float xl = tf(x[(((long)img * a.H + hc) * a.W + wc) * a.C + cc[j]]);
            xv[j] = in ? xl : 0.f;
        }
#pragma unroll
        for (int v = 0; v < KT / VEC; ++v) {
            const Vec d = *(const Vec *)(dy + (long)l * KT + v * VEC);   // the same address in all column lanes
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const float df = tf(d[e]);
                acc[0][v * VEC + e] += df * xv[0];
                acc[1][v * VEC + e] += df * xv[1];
            }
        }
        q += PL;
        while (q >= a.Q) {
            q -= a.Q;
            if (++p == a.P) {
                p = 0;
                ++img;
            }
        }
    }
    // combine the pixel lanes, 16 output channels at a time, in a fixed order
    float *__restrict__ part = a.part + (long)split * KT * NT;   // [KT][NT]
#pragma unroll
    for (int k0 = 0; k0 < KT; k0 += 16) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int k = 0; k < 16; ++k) red[(pl * 16 + k) * COLS + 2 * lc + j] = acc[j][k0 + k];
        __syncthreads();
        // 512 sums of this round: thread -> (k = tid / 32 and + 8, column)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int k = tid / COLS + kk * 8, cl = tid % COLS;
            float s = 0.f;
#pragma unroll
            for (int r = 0; r < PL; ++r) s += red[(r * 16 + k) * COLS + cl];
            const int ocol = blockIdx.x * COLS + cl;
            if (ocol < NT) part[(long)(k0 + k) * NT + ocol] = s;
        }
        __syncthreads();
    }
}

bool al16(const void *p) { return ((uintptr_t)p & 15) == 0; }
bool tiny_off() { return hooks().no_tiny; }   // test hook

}  // namespace

bool tiny_src_applicable(int dtype, const IgemmArgs &a)
{
    const int vec = dtype == NSK_BF16 ? 8 : 4;
    if (tiny_off() || a.groups > 1 || a.stats || a.zero_cell) return false;
    if (a.Cs < 1 || a.Cs > TINY_MAX_C || a.Ktot != a.ntaps * a.Cs) return false;
    if (!(a.Ngemm == 8 || a.Ngemm == 16 || a.Ngemm == 32 || a.Ngemm == 64) || a.Ngemm % vec != 0) return false;
    return a.Co % vec == 0 && al16(a.out) && (long)a.Ktot * a.Ngemm * 4 <= TINY_LDS_MAX;
}

int launch_tiny_src(int dtype, const IgemmArgs &a, hipStream_t stream)
{
    const dim3 grid(ceil_div(ceil_div(a.M, TINY_PIX), 256)), block(256);
    const size_t lds = (size_t)a.Ktot * a.Ngemm * sizeof(float);
#define NSK_TINY_SRC(T, NG) hipLaunchKernelGGL((tiny_src_kernel<T, NG>), grid, block, lds, stream, a)
    if (dtype == NSK_BF16) {
        switch (a.Ngemm) {
        case 8: NSK_TINY_SRC(bf16_t, 8); break;
        case 16: NSK_TINY_SRC(bf16_t, 16); break;
        case 32: NSK_TINY_SRC(bf16_t, 32); break;
        default: NSK_TINY_SRC(bf16_t, 64); break;
        }
    } else {
        switch (a.Ngemm) {
        case 8: NSK_TINY_SRC(float, 8); break;
        case 16: NSK_TINY_SRC(float, 16); break;
        case 32: NSK_TINY_SRC(float, 32); break;
        default: NSK_TINY_SRC(float, 64); break;
        }
    }
#undef NSK_TINY_SRC
    return check_launch();
}

bool tiny_out_applicable(int dtype, const IgemmArgs &a)
{
    if (tiny_off() || a.groups > 1 || a.stats || a.zero_cell) return false;
    if (a.Ngemm < 1 || a.Ngemm > TINY_MAX_C || a.Ktot != a.ntaps * a.Cs) return false;
    if (!(a.Cs == 16 || a.Cs == 32 || a.Cs == 64)) return false;
    return al16(a.src) && (long)a.ntaps * TINY_MAX_C * a.Cs * 4 <= TINY_LDS_MAX;
}

int launch_tiny_out(int dtype, const IgemmArgs &a, hipStream_t stream)
{
    const dim3 grid(ceil_div(a.M, 256)), block(256);
    const size_t lds = (size_t)a.ntaps * TINY_MAX_C * a.Cs * (dtype == NSK_BF16 ? 2 : 4);
#define NSK_TINY_OUT(T, CS) hipLaunchKernelGGL((tiny_out_kernel<T, CS>), grid, block, lds, stream, a)
    if (dtype == NSK_BF16) {
        if (a.Cs == 16) NSK_TINY_OUT(bf16_t, 16);
        else if (a.Cs == 32) NSK_TINY_OUT(bf16_t, 32);
        else NSK_TINY_OUT(bf16_t, 64);
    } else {
        if (a.Cs == 16) NSK_TINY_OUT(float, 16);
        else if (a.Cs == 32) NSK_TINY_OUT(float, 32);
        else NSK_TINY_OUT(float, 64);
    }
#undef NSK_TINY_OUT
    return check_launch();
}

bool tiny_wgrad_applicable(int dtype, const WgradArgs &a)
{
    if (tiny_off() || a.groups > 1) return false;
    if (a.C < 1 || a.C > TINY_MAX_C) return false;
    if (!(a.K == 16 || a.K == 32 || a.K == 64)) return false;
    return al16(a.dy) && a.splits >= 1 && a.splits <= 65535;
}

int launch_tiny_wgrad(int dtype, const WgradArgs &a, hipStream_t stream)
{
    const dim3 grid(ceil_div(a.ntaps * a.C, 32), a.splits), block(256);
#define NSK_TINY_WG(T, KT) hipLaunchKernelGGL((tiny_wgrad_kernel<T, KT>), grid, block, 0, stream, a)
    if (dtype == NSK_BF16) {
        if (a.K == 16) NSK_TINY_WG(bf16_t, 16);
        else if (a.K == 32) NSK_TINY_WG(bf16_t, 32);
        else NSK_TINY_WG(bf16_t, 64);
    } else {
        if (a.K == 16) NSK_TINY_WG(float, 16);
        else if (a.K == 32) NSK_TINY_WG(float, 32);
        else NSK_TINY_WG(float, 64);
    }
#undef NSK_TINY_WG
    return check_launch();
}

}  // namespace nsk

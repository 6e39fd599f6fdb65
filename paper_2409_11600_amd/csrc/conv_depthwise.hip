// Depthwise convolution (a grouped convolution with one input and one output channel per group; the grouped entry
// points of the library, not one of the paper's workloads): y[n][p][q][c] = sum over taps of x[n][h][w][c] * w[c][tap].
// There is no contraction over channels, so nothing here is GEMM-shaped: every pass reads each activation once from
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
#include "nsk_internal.h"

namespace nsk {
namespace {

constexpr int DW_PIX = 4;          // output pixels per lane (forward / backward-data)
constexpr int DW_LDS_MAX = 48 << 10;  // bytes of LDS the transposed filter may take
constexpr int DW_TC = 9;           // taps per register chunk of the backward-weight kernel
constexpr int DW_CVB = 16;         // channel vectors per backward-weight block

template <typename T> struct DTraits;
template <> struct DTraits<float> {
    static constexpr int VEC = 4;
    typedef f32x4 Vec;
};
template <> struct DTraits<bf16_t> {
    static constexpr int VEC = 8;
    typedef bf16x8 Vec;
};

template <typename T>
__global__ __launch_bounds__(256) void depthwise_kernel(const IgemmArgs a)
{
    typedef typename DTraits<T>::Vec Vec;
    constexpr int VEC = DTraits<T>::VEC;
    extern __shared__ __attribute__((aligned(16))) float wT[];   // [ntaps][C]
    __shared__ short s_offh[kMaxTaps], s_offw[kMaxTaps];
    const int tid = threadIdx.x;
    const int C = a.groups, CV = C / VEC, ntaps = a.ntaps;
    const T *__restrict__ src = (const T *)a.src;
    const T *__restrict__ wpk = (const T *)a.wpk;      // [C][ntaps]
    T *__restrict__ out = (T *)a.out;
    for (int i = tid; i < ntaps * C; i += 256) {
        const int c = i / ntaps, t = i - c * ntaps;
        wT[t * C + c] = (float)wpk[i];
    }
    if (tid < kMaxTaps) {
        s_offh[tid] = a.off_h[tid];
        s_offw[tid] = a.off_w[tid];
    }
    __syncthreads();

    const long f = (long)blockIdx.x * 256 + tid;
    const int cv = (int)(f % CV);
    const long slot = f / CV;
    if (slot * DW_PIX >= a.M) return;
    const int c0 = cv * VEC;

    bool ok[DW_PIX];
    int bh[DW_PIX], bw[DW_PIX];
    long src_img[DW_PIX], out_off[DW_PIX];
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
        src_img[u] = (long)img * a.Hs;
        out_off[u] = (((long)img * a.Ho + (i * a.osh + a.oa)) * a.Wo + (j * a.osw + a.ob)) * C + c0;
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[u][e] = 0.f;
        if (a.accumulate && ok[u]) {   // start from the old values: the sum is rounded to the storage type once
            const Vec old = *(const Vec *)(out + out_off[u]);
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[u][e] = (float)old[e];
        }
    }
    for (int t = 0; t < ntaps; ++t) {
        float wv[VEC];
#pragma unroll
        for (int e = 0; e < VEC; e += 4) {
            const f32x4 q = *(const f32x4 *)&wT[t * C + c0 + e];
            wv[e] = q[0]; wv[e + 1] = q[1]; wv[e + 2] = q[2]; wv[e + 3] = q[3];
        }
        const int oh = s_offh[t], ow = s_offw[t];
#pragma unroll
        for (int u = 0; u < DW_PIX; ++u) {
            const int h = bh[u] + oh, w = bw[u] + ow;
            if (ok[u] && (unsigned)h < (unsigned)a.Hs && (unsigned)w < (unsigned)a.Ws) {
                const Vec xv = *(const Vec *)(src + ((src_img[u] + h) * a.Ws + w) * C + c0);
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[u][e] += (float)xv[e] * wv[e];
            }
        }
    }
#pragma unroll
    for (int u = 0; u < DW_PIX; ++u) {
        if (!ok[u]) continue;
        Vec o;
#pragma unroll
        for (int e = 0; e < VEC; ++e) o[e] = (T)acc[u][e];
        *(Vec *)(out + out_off[u]) = o;
    }
}

template <typename T>
__global__ __launch_bounds__(256) void depthwise_wgrad_kernel(const WgradArgs a)
{
    typedef typename DTraits<T>::Vec Vec;
    constexpr int VEC = DTraits<T>::VEC;
    __shared__ float red[256 * VEC];
    __shared__ short s_offh[kMaxTaps], s_offw[kMaxTaps];
    const int tid = threadIdx.x;
    const int C = a.groups, CV = C / VEC;
    const int cvb = min(CV - (int)blockIdx.x * DW_CVB, DW_CVB);   // channel vectors of this block (>= 1)
    const int PL = 256 / cvb;                                     // pixel lanes
    const int cvl = tid % cvb, pl = tid / cvb;
    const bool active = pl < PL;
    const int c0 = (blockIdx.x * DW_CVB + cvl) * VEC;
    const int split = blockIdx.y;
    const T *__restrict__ x = (const T *)a.x;
    const T *__restrict__ dy = (const T *)a.dy;
    if (tid < kMaxTaps) {
        s_offh[tid] = a.off_h[tid];
        s_offw[tid] = a.off_w[tid];
    }
    __syncthreads();
    const int l_begin = split * a.rows_per_split;
    const int l_end = min(a.L, l_begin + a.rows_per_split);
    const int pq = a.P * a.Q;
    float *__restrict__ part = a.part + (long)split * C * a.ntaps;   // [C][ntaps]

    for (int t0 = 0; t0 < a.ntaps; t0 += DW_TC) {
        float acc[DW_TC][VEC];
#pragma unroll
        for (int tt = 0; tt < DW_TC; ++tt)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[tt][e] = 0.f;
        if (active)
            for (int l = l_begin + pl; l < l_end; l += PL) {
                const int img = l / pq;
                const int rem = l - img * pq;
                const int p = rem / a.Q;
                const int q = rem - p * a.Q;
                const Vec dv = *(const Vec *)(dy + (long)l * C + c0);
                float df[VEC];
#pragma unroll
                for (int e = 0; e < VEC; ++e) df[e] = (float)dv[e];
                const int h0 = p * a.sh - a.ph, w0 = q * a.sw - a.pw;
#pragma unroll
                for (int tt = 0; tt < DW_TC; ++tt) {
                    const int t = t0 + tt;
                    if (t >= a.ntaps) break;
                    const int h = h0 + s_offh[t], w = w0 + s_offw[t];
                    if ((unsigned)h < (unsigned)a.H && (unsigned)w < (unsigned)a.W) {
                        const Vec xv = *(const Vec *)(x + (((long)img * a.H + h) * a.W + w) * C + c0);
#pragma unroll
                        for (int e = 0; e < VEC; ++e) acc[tt][e] += df[e] * (float)xv[e];
                    }
                }
            }
        // combine the pixel lanes, one tap at a time, in a fixed order
#pragma unroll
        for (int tt = 0; tt < DW_TC; ++tt) {
            const int t = t0 + tt;
            if (t >= a.ntaps) break;    // uniform over the block
            if (active)
#pragma unroll
                for (int e = 0; e < VEC; ++e) red[pl * (cvb * VEC) + cvl * VEC + e] = acc[tt][e];
            __syncthreads();
            if (tid < cvb * VEC) {
                float s = 0.f;
                for (int r = 0; r < PL; ++r) s += red[r * (cvb * VEC) + tid];
                const int c = blockIdx.x * DW_CVB * VEC + tid;
                part[(long)c * a.ntaps + t] = s;
            }
            __syncthreads();
        }
    }
}

bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace

bool depthwise_applicable(int dtype, const IgemmArgs &a)
{
    const int vec = dtype == NSK_BF16 ? 8 : 4;
    return a.groups > 1 && a.Cs == 1 && a.Ngemm == 1 && a.src_ld == a.groups && a.Co == a.groups &&
           a.groups % vec == 0 && (long)a.ntaps * a.groups * 4 <= DW_LDS_MAX && a.ntaps >= 1 && !a.stats &&
           aligned16(a.src) && aligned16(a.out);
}

int launch_depthwise(int dtype, const IgemmArgs &a, hipStream_t stream)
{
    const int vec = dtype == NSK_BF16 ? 8 : 4;
    const long threads = ((long)a.M + DW_PIX - 1) / DW_PIX * (a.groups / vec);
    const unsigned blocks = (unsigned)((threads + 255) / 256);
    const size_t lds = (size_t)a.ntaps * a.groups * sizeof(float);
    if (dtype == NSK_BF16)
        hipLaunchKernelGGL((depthwise_kernel<bf16_t>), dim3(blocks), dim3(256), lds, stream, a);
    else
        hipLaunchKernelGGL((depthwise_kernel<float>), dim3(blocks), dim3(256), lds, stream, a);
    return check_launch();
}

bool depthwise_wgrad_applicable(int dtype, const WgradArgs &a)
{
    const int vec = dtype == NSK_BF16 ? 8 : 4;
    return a.groups > 1 && a.C == 1 && a.K == 1 && a.ldx == a.groups && a.ldy == a.groups && a.groups % vec == 0 &&
           a.splits >= 1 && a.splits <= 65535 && aligned16(a.x) && aligned16(a.dy);
}

int launch_depthwise_wgrad(int dtype, const WgradArgs &a, hipStream_t stream)
{
    const int vec = dtype == NSK_BF16 ? 8 : 4;
    dim3 grid(ceil_div(a.groups / vec, DW_CVB), a.splits);
    if (dtype == NSK_BF16)
        hipLaunchKernelGGL((depthwise_wgrad_kernel<bf16_t>), grid, dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL((depthwise_wgrad_kernel<float>), grid, dim3(256), 0, stream, a);
    return check_launch();
}

}  // namespace nsk

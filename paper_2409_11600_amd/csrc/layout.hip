// Layout helpers at the library boundary: the kernels compute in NHWC / "filter row = all taps of
// one output channel"; callers that hold NCHW / KCRS tensors are served by these copies through
// the workspace.  Pure data movement, bounded by HBM bandwidth.
#include "nsk_internal.h"

namespace nsk {
namespace {

// Per image: src [rows][cols] -> dst [cols][rows], 32x32 tiles through LDS (padded by one
// column so the transposed reads are conflict-free).  accumulate adds into dst.
template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T *__restrict__ src, T *__restrict__ dst, int rows,
                                                        int cols, int accumulate)
{
    __shared__ float tile[32][33];
    const long img = blockIdx.z;
    src += img * rows * cols;
    dst += img * rows * cols;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
#pragma unroll
    for (int i = 0; i < 32; i += 8) {
        const int r = r0 + ty + i, c = c0 + tx;
        if (r < rows && c < cols) tile[ty + i][tx] = (float)src[(long)r * cols + c];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 32; i += 8) {
        const int c = c0 + ty + i, r = r0 + tx;
        if (r < rows && c < cols) {
            float v = tile[tx][ty + i];
            T *o = dst + (long)c * rows + r;
            if (accumulate) v += (float)*o;
            *o = (T)v;
        }
    }
}

struct PackArgs {
    const void *w;
    void *out;
    int Nn, ntaps, Cs;
    long sn, sc;
    long w_gstep;   // grouped filters: blockIdx.z names the group, whose source lies w_gstep elements further
    int tap_off[kMaxTaps];
};

// Up to four packings in one launch (blockIdx.y names the packing): the residue classes of a strided backward-data
// pass each need their own packed filter, and a launch per class costs more than the copy.
constexpr int kPackMulti = 4;
struct PackMulti {
    PackArgs e[kPackMulti];
};

template <typename T> __global__ __launch_bounds__(256) void pack_filter_kernel(const PackMulti m)
{
    const PackArgs &a = m.e[blockIdx.y];
    const long total = (long)a.Nn * a.ntaps * a.Cs;
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int c = (int)(i % a.Cs);
    const long r = i / a.Cs;
    const int t = (int)(r % a.ntaps);
    const long n = r / a.ntaps;
    const long g = blockIdx.z;
    ((T *)a.out)[g * total + i] = ((const T *)a.w)[g * a.w_gstep + n * a.sn + a.tap_off[t] + c * a.sc];
}

// Zero the pixels (i*osh + oa, j*osw + ob), i < Mi, j < Mj, of every image of an NHWC tensor: the cells
// of a strided backward-data result that no filter tap reaches.  `unit` = bytes written per thread.
__global__ __launch_bounds__(256) void zero_class_kernel(unsigned char *__restrict__ out, long total, int Mi, int Mj, int Ho,
                                                         int Wo, int osh, int oa, int osw, int ob, int pix_bytes,
                                                         int unit)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int upp = pix_bytes / unit;            // units per pixel
    const int u = (int)(i % upp);
    long r = i / upp;
    const int j = (int)(r % Mj); r /= Mj;
    const int ii = (int)(r % Mi);
    const long img = r / Mi;
    unsigned char *p = out + ((img * Ho + (ii * osh + oa)) * Wo + (j * osw + ob)) * (long)pix_bytes + (long)u * unit;
    if (unit == 16) *(f32x4 *)p = f32x4{0.f, 0.f, 0.f, 0.f};
    else if (unit == 4) *(float *)p = 0.f;
    else *(unsigned short *)p = 0;
}

template <typename T>
int transpose_typed(const void *src, void *dst, int batch, int rows, int cols, int accumulate, hipStream_t stream)
{
    dim3 grid(ceil_div(cols, 32), ceil_div(rows, 32), batch);
    hipLaunchKernelGGL((transpose_kernel<T>), grid, dim3(256), 0, stream, (const T *)src, (T *)dst, rows, cols,
                       accumulate);
    return check_launch();
}

}  // namespace

int launch_nchw_to_nhwc(int dtype, const void *src, void *dst, int N, int C, int H, int W, hipStream_t stream)
{
    if (dtype == NSK_BF16) return transpose_typed<bf16_t>(src, dst, N, C, H * W, 0, stream);
    return transpose_typed<float>(src, dst, N, C, H * W, 0, stream);
}

int launch_nhwc_to_nchw(int dtype, const void *src, void *dst, int N, int C, int H, int W, int accumulate,
                        hipStream_t stream)
{
    if (dtype == NSK_BF16) return transpose_typed<bf16_t>(src, dst, N, H * W, C, accumulate, stream);
    return transpose_typed<float>(src, dst, N, H * W, C, accumulate, stream);
}

int launch_zero_class(int dtype, void *out, int Nimg, int Ho, int Wo, int Co, int Mi, int Mj, int osh, int oa, int osw,
                      int ob, hipStream_t stream)
{
    const int pix_bytes = Co * (int)elem_size(dtype);
    const int unit = pix_bytes % 16 == 0 ? 16 : (pix_bytes % 4 == 0 ? 4 : 2);
    const long total = (long)Nimg * Mi * Mj * (pix_bytes / unit);
    if (total == 0) return NSK_OK;
    hipLaunchKernelGGL(zero_class_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, (unsigned char *)out,
                       total, Mi, Mj, Ho, Wo, osh, oa, osw, ob, pix_bytes, unit);
    return check_launch();
}

int launch_pack_filters(int dtype, int count, const void *w, void *const *out, int Nn, const int *ntaps, int Cs, long sn,
                        long sc, const int (*tap_off_host)[kMaxTaps], hipStream_t stream)
{
    return launch_pack_filters_grouped(dtype, count, w, out, Nn, ntaps, Cs, sn, sc, tap_off_host, 1, 0L, stream);
}

int launch_pack_filters_grouped(int dtype, int count, const void *w, void *const *out, int Nn, const int *ntaps, int Cs,
                                long sn, long sc, const int (*tap_off_host)[kMaxTaps], int groups, long w_gstep,
                                hipStream_t stream)
{
    if (count < 1 || count > kPackMulti || groups < 1 || groups > 65535) return NSK_ERR_BAD_DESC;
    PackMulti m{};
    long most = 0;
    for (int k = 0; k < count; ++k) {
        PackArgs &a = m.e[k];
        a.w = w;
        a.out = out[k];
        a.Nn = Nn;
        a.ntaps = ntaps[k];
        a.Cs = Cs;
        a.sn = sn;
        a.sc = sc;
        a.w_gstep = w_gstep;
        for (int t = 0; t < kMaxTaps; ++t) a.tap_off[t] = t < ntaps[k] ? tap_off_host[k][t] : 0;
        const long total = (long)Nn * ntaps[k] * Cs;
        if (total > most) most = total;
    }
    if (most == 0) return NSK_OK;
    dim3 grid((unsigned)((most + 255) / 256), (unsigned)count, (unsigned)groups);
    if (dtype == NSK_BF16)
        hipLaunchKernelGGL((pack_filter_kernel<bf16_t>), grid, dim3(256), 0, stream, m);
    else
        hipLaunchKernelGGL((pack_filter_kernel<float>), grid, dim3(256), 0, stream, m);
    return check_launch();
}

int launch_pack_filter(int dtype, const void *w, void *out, int Nn, int ntaps, int Cs, long sn, long sc,
                       const int *tap_off_host, hipStream_t stream)
{
    int taps[1][kMaxTaps];
    for (int t = 0; t < kMaxTaps; ++t) taps[0][t] = t < ntaps ? tap_off_host[t] : 0;
    void *outs[1] = {out};
    return launch_pack_filters(dtype, 1, w, outs, Nn, &ntaps, Cs, sn, sc, taps, stream);
}

}  // namespace nsk

// The recurrent workload of the paper (section "Experiments and Discussion": embedding over the vocabulary, one GRU
// layer of hidden size 256, an output layer, cross entropy, AdamW): the pieces that are not matrix products.  The
// products (x @ W_ih for all time steps at once, h @ W_hh per step, and their gradients) are the `@` operator
// (nsk_linear_*); here are the embedding lookup with its gradient and the fused elementwise part of a GRU step in
// both directions.  The paper ran these as separate unfused operations and names that as the reason for its 15x
// slowdown on this experiment; one kernel per direction replaces about a dozen elementwise launches per step.
//
// Gate convention (of the framework the paper compares against): with gi = x @ W_ih and gh = h @ W_hh, gates (r, z, n),
//   r = sigmoid(gi_r + b_ir + gh_r + b_hr),  z = sigmoid(gi_z + b_iz + gh_z + b_hz),
//   q = gh_n + b_hn,  n = tanh(gi_n + b_in + r*q),  h' = (1 - z)*n + z*h.
#include <math.h>

#include "nsk_internal.h"

namespace nsk {
namespace {

bool unaligned16(const void *p) { return ((uintptr_t)p & 15) != 0; }
bool dtype_ok(int dtype) { return dtype == NSK_F32 || dtype == NSK_BF16; }

__device__ inline float ld(const float *p, long i) { return p[i]; }
__device__ inline float ld(const bf16_t *p, long i) { return (float)p[i]; }
__device__ inline float sigmoidf(float a) { return 1.f / (1.f + expf(-a)); }

// ----------------------------------------------------------------------------- embedding
template <typename T>
__global__ __launch_bounds__(256) void embedding_fwd_kernel(const int *__restrict__ tokens, const T *__restrict__ table,
                                                            T *__restrict__ out, long total, int E, int V)
{
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const long row = i / E;
        const int e = (int)(i - row * E), v = tokens[row];
        out[i] = (v >= 0 && v < V) ? table[(long)v * E + e] : (T)NAN;
    }
}

// Gradient of the lookup without atomics: block b owns the vocabulary rows v with v % gridDim.x == b, walks over ALL
// positions in order and adds the rows that are its own, so every dtable element is updated by one thread in
// position order (bitwise reproducible).  The token list is tiny next to the table, every block reads all of it.
template <typename T>
__global__ __launch_bounds__(256) void embedding_bwd_kernel(const int *__restrict__ tokens, const T *__restrict__ dout,
                                                            float *__restrict__ dtable, int n, int E, int V, int accumulate)
{
    __shared__ int hit[256];         // positions of this chunk whose row belongs to the block, in position order
    __shared__ int wave_hits[4];
    const int b = blockIdx.x, nb = gridDim.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (!accumulate)
        for (int v = b; v < V; v += nb)
            for (int e = threadIdx.x; e < E; e += 256) dtable[(long)v * E + e] = 0.f;
    for (int base = 0; base < n; base += 256) {
        // all 256 positions of the chunk are tested at once; the matches are compacted in position order
        const int i = base + threadIdx.x;
        const int v = i < n ? tokens[i] : -1;
        const bool mine = v >= 0 && v < V && v % nb == b;
        const unsigned long long ballot = __ballot(mine);
        if (lane == 0) wave_hits[wave] = __popcll(ballot);
        __syncthreads();
        int before = 0;
        for (int w = 0; w < wave; ++w) before += wave_hits[w];
        const int total = wave_hits[0] + wave_hits[1] + wave_hits[2] + wave_hits[3];
        if (mine) hit[before + __popcll(ballot & ((1ull << lane) - 1ull))] = i;
        __syncthreads();
        for (int k = 0; k < total; ++k) {
            const int pos = hit[k];
            const long row = (long)tokens[pos] * E;
            for (int e = threadIdx.x; e < E; e += 256) dtable[row + e] += ld(dout, (long)pos * E + e);
        }
        __syncthreads();
    }
}

// ----------------------------------------------------------------------------- GRU step, elementwise part
template <typename T>
__global__ __launch_bounds__(256) void gru_gates_fwd_kernel(const T *__restrict__ gi, const T *__restrict__ gh,
                                                            const float *__restrict__ b_ih, const float *__restrict__ b_hh,
                                                            const T *__restrict__ h_prev, T *__restrict__ h_new,
                                                            T *__restrict__ saved, long total, int H)
{
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const long n = i / H;
        const int h = (int)(i - n * H);
        const long g0 = n * 3 * H + h;
        const float r = sigmoidf(ld(gi, g0) + b_ih[h] + ld(gh, g0) + b_hh[h]);
        const float z = sigmoidf(ld(gi, g0 + H) + b_ih[H + h] + ld(gh, g0 + H) + b_hh[H + h]);
        const float q = ld(gh, g0 + 2 * H) + b_hh[2 * H + h];
        const float c = tanhf(ld(gi, g0 + 2 * H) + b_ih[2 * H + h] + r * q);
        h_new[i] = (T)((1.f - z) * c + z * ld(h_prev, i));
        T *s = saved + n * 4 * H + h;
        s[0] = (T)r;
        s[H] = (T)z;
        s[2 * H] = (T)c;
        s[3 * H] = (T)q;
    }
}

template <typename T>
__global__ __launch_bounds__(256) void gru_gates_bwd_kernel(const T *__restrict__ saved, const T *__restrict__ h_prev,
                                                            const T *__restrict__ dh_a, const T *__restrict__ dh_b,
                                                            const T *__restrict__ dh_c, T *__restrict__ dgi,
                                                            T *__restrict__ dgh, T *__restrict__ dh_direct, long total, int H)
{
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const long n = i / H;
        const int h = (int)(i - n * H);
        const T *s = saved + n * 4 * H + h;
        const float r = ld(s, 0), z = ld(s, H), c = ld(s, 2 * H), q = ld(s, 3 * H);
        float dh = ld(dh_a, i);
        if (dh_b) dh += ld(dh_b, i);
        if (dh_c) dh += ld(dh_c, i);
        const float da_n = dh * (1.f - z) * (1.f - c * c);
        const float da_z = dh * (ld(h_prev, i) - c) * z * (1.f - z);
        const float da_r = da_n * q * r * (1.f - r);
        const long g0 = n * 3 * H + h;
        dgi[g0] = (T)da_r;
        dgi[g0 + H] = (T)da_z;
        dgi[g0 + 2 * H] = (T)da_n;
        dgh[g0] = (T)da_r;
        dgh[g0 + H] = (T)da_z;
        dgh[g0 + 2 * H] = (T)(da_n * r);
        dh_direct[i] = (T)(dh * z);
    }
}

// ----------------------------------------------------------------------------- GRU step, product and gates in one kernel
// With a few dozen rows the recurrent product h @ W_hh is a 20 MFLOP launch of its own followed by the gate kernel,
// 400 dependent launches for 200 time steps.  Here block (u, chunk) owns hidden unit u for a chunk of the samples; L
// neighbouring lanes (sample n, part q) split each of the unit's dot products (three of length H forward, one of
// length 3H with the gradients of the step after backward: q takes every L-th 16-byte vector, so the L lanes read
// contiguous bytes of the sample's row, and all lanes with the same q read the same weight vector), add up their parts
// in a fixed order, and lane q = 0 goes straight on to the gate arithmetic of (n, u).  L is chosen so that a lane's
// loads are few enough to be in flight all at once: the kernel is one L2 round trip and a store.  No LDS, no
// barrier; gh is never stored.
__device__ inline f32x4 ld4(const float *p) { return *(const f32x4 *)p; }
__device__ inline f32x4 ld4(const bf16_t *p)
{
    const bf16x4 v = *(const bf16x4 *)p;
    return f32x4{(float)v[0], (float)v[1], (float)v[2], (float)v[3]};
}
template <int L> __device__ inline float lanes_sum(const f32x4 a)
{
    float s = (a[0] + a[1]) + (a[2] + a[3]);
#pragma unroll
    for (int o = 1; o < L; o <<= 1) s += __shfl_xor(s, o, 64);
    return s;
}
constexpr int GS_THREADS = 512, GS_LF = 8, GS_LB = 16;   // lanes per dot product, forward and backward

template <typename T>
__global__ __launch_bounds__(GS_THREADS) void gru_step_fwd_kernel(const T *__restrict__ gi, const T *__restrict__ w_hh,
                                                           const float *__restrict__ b_ih, const float *__restrict__ b_hh,
                                                           const T *__restrict__ h_prev, T *__restrict__ h_new,
                                                           T *__restrict__ saved, int N, int H)
{
    constexpr int L = GS_LF, SLOTS = GS_THREADS / L;
    const int u = blockIdx.x, q = threadIdx.x & (L - 1), slot = threadIdx.x / L, H4 = H >> 2;
    const T *w0 = w_hh + (long)u * H, *w1 = w0 + (long)H * H, *w2 = w1 + (long)H * H;   // rows u, H + u, 2H + u
    {
        const int n0 = blockIdx.y * SLOTS;
        const int n = n0 + slot < N ? n0 + slot : N - 1;   // lanes past the end repeat the last sample and store nothing
        const T *hp = h_prev + (long)n * H;
        // the gate operands are requested before the dot products, so that the kernel is one round trip, not two
        const long g0 = (long)n * 3 * H + u;
        const float gi_r = ld(gi, g0), gi_z = ld(gi, g0 + H), gi_n = ld(gi, g0 + 2 * H), h_old = ld(h_prev, (long)n * H + u);
        const float br = b_ih[u] + b_hh[u], bz = b_ih[H + u] + b_hh[H + u], bin = b_ih[2 * H + u], bhn = b_hh[2 * H + u];
        f32x4 a0 = {0.f, 0.f, 0.f, 0.f}, a1 = a0, a2 = a0;
        // (unrolled so that the loads of several vectors are in flight together: each is an L2 round trip)
#pragma unroll 8
        for (int j4 = q; j4 < H4; j4 += L) {
            const f32x4 h4 = ld4(hp + 4 * j4);
            a0 += h4 * ld4(w0 + 4 * j4);
            a1 += h4 * ld4(w1 + 4 * j4);
            a2 += h4 * ld4(w2 + 4 * j4);
        }
        const float gh_r = lanes_sum<L>(a0), gh_z = lanes_sum<L>(a1), gh_n = lanes_sum<L>(a2);
        if (q != 0 || n0 + slot >= N) return;
        const float r = sigmoidf(gi_r + gh_r + br);
        const float z = sigmoidf(gi_z + gh_z + bz);
        const float qq = gh_n + bhn;
        const float c = tanhf(gi_n + bin + r * qq);
        h_new[(long)n * H + u] = (T)((1.f - z) * c + z * h_old);
        T *sv = saved + (long)n * 4 * H + u;
        sv[0] = (T)r;
        sv[H] = (T)z;
        sv[2 * H] = (T)c;
        sv[3 * H] = (T)qq;
    }
}

template <typename T>
__global__ __launch_bounds__(GS_THREADS) void gru_step_bwd_kernel(const T *__restrict__ saved, const T *__restrict__ h_prev,
                                                           const T *__restrict__ dh_a, const T *__restrict__ dh_direct_next,
                                                           const T *__restrict__ dgh_next, const T *__restrict__ w_hh_t,
                                                           T *__restrict__ dgi, T *__restrict__ dgh, T *__restrict__ dh_direct,
                                                           int N, int H)
{
    constexpr int L = GS_LB, SLOTS = GS_THREADS / L;
    const int u = blockIdx.x, q = threadIdx.x & (L - 1), slot = threadIdx.x / L, J = 3 * H, J4 = J >> 2;
    const T *wt = w_hh_t + (long)u * J;   // column u of W_hh
    {
        const int n0 = blockIdx.y * SLOTS;
        const int n = n0 + slot < N ? n0 + slot : N - 1;
        // the elementwise operands are requested before the dot product (one round trip, not two)
        const long i = (long)n * H + u;
        const T *sv = saved + (long)n * 4 * H + u;
        const float r = ld(sv, 0), z = ld(sv, H), c = ld(sv, 2 * H), qq = ld(sv, 3 * H), h_old = ld(h_prev, i);
        const float dh_other = (dh_direct_next ? ld(dh_direct_next, i) : 0.f) + (dh_a ? ld(dh_a, i) : 0.f);
        float dh = 0.f;
        if (dgh_next) {   // the part of the gradient that came back through the recurrent product of the step after
            const T *d = dgh_next + (long)n * J;
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 12
            for (int j4 = q; j4 < J4; j4 += L) acc += ld4(d + 4 * j4) * ld4(wt + 4 * j4);
            dh = lanes_sum<L>(acc);
        }
        if (q != 0 || n0 + slot >= N) return;
        dh += dh_other;
        const float da_n = dh * (1.f - z) * (1.f - c * c);
        const float da_z = dh * (h_old - c) * z * (1.f - z);
        const float da_r = da_n * qq * r * (1.f - r);
        const long g0 = (long)n * J + u;
        dgi[g0] = (T)da_r;
        dgi[g0 + H] = (T)da_z;
        dgi[g0 + 2 * H] = (T)da_n;
        dgh[g0] = (T)da_r;
        dgh[g0 + H] = (T)da_z;
        dgh[g0 + 2 * H] = (T)(da_n * r);
        dh_direct[i] = (T)(dh * z);
    }
}

int grid_for(long items)
{
    long b = (items + 255) / 256;
    if (b > 4096) b = 4096;
    return (int)(b < 1 ? 1 : b);
}

}  // namespace
}  // namespace nsk

using namespace nsk;

extern "C" {

int nsk_embedding_fwd(int dtype, int n, int E, int V, const int *tokens, const void *table, void *out, void *stream)
{
    if (n <= 0 || E <= 0 || V <= 0 || !dtype_ok(dtype)) return NSK_ERR_BAD_DESC;
    if (!tokens || !table || !out) return NSK_ERR_NULL;
    if (unaligned16(tokens) || unaligned16(table) || unaligned16(out)) return NSK_ERR_ALIGNMENT;
    const long total = (long)n * E;
    if (dtype == NSK_BF16)
        hipLaunchKernelGGL(embedding_fwd_kernel<bf16_t>, dim3(grid_for(total)), dim3(256), 0, (hipStream_t)stream, tokens,
                           (const bf16_t *)table, (bf16_t *)out, total, E, V);
    else
        hipLaunchKernelGGL(embedding_fwd_kernel<float>, dim3(grid_for(total)), dim3(256), 0, (hipStream_t)stream, tokens,
                           (const float *)table, (float *)out, total, E, V);
    return check_launch();
}

int nsk_embedding_bwd(int dtype, int n, int E, int V, const int *tokens, const void *dout, float *dtable, int accumulate,
                      void *stream)
{
    if (n <= 0 || E <= 0 || V <= 0 || !dtype_ok(dtype) || (accumulate != 0 && accumulate != 1)) return NSK_ERR_BAD_DESC;
    if (!tokens || !dout || !dtable) return NSK_ERR_NULL;
    if (unaligned16(tokens) || unaligned16(dout) || unaligned16(dtable)) return NSK_ERR_ALIGNMENT;
    const int blocks = V < 1024 ? V : 1024;
    if (dtype == NSK_BF16)
        hipLaunchKernelGGL(embedding_bwd_kernel<bf16_t>, dim3(blocks), dim3(256), 0, (hipStream_t)stream, tokens,
                           (const bf16_t *)dout, dtable, n, E, V, accumulate);
    else
        hipLaunchKernelGGL(embedding_bwd_kernel<float>, dim3(blocks), dim3(256), 0, (hipStream_t)stream, tokens,
                           (const float *)dout, dtable, n, E, V, accumulate);
    return check_launch();
}

int nsk_gru_gates_fwd(int dtype, int N, int H, const void *gi, const void *gh, const float *b_ih, const float *b_hh,
                      const void *h_prev, void *h_new, void *saved, void *stream)
{
    if (N <= 0 || H <= 0 || !dtype_ok(dtype)) return NSK_ERR_BAD_DESC;
    if (!gi || !gh || !b_ih || !b_hh || !h_prev || !h_new || !saved) return NSK_ERR_NULL;
    if (unaligned16(gi) || unaligned16(gh) || unaligned16(b_ih) || unaligned16(b_hh) || unaligned16(h_prev) ||
        unaligned16(h_new) || unaligned16(saved))
        return NSK_ERR_ALIGNMENT;
    const long total = (long)N * H;
    if (dtype == NSK_BF16)
        hipLaunchKernelGGL(gru_gates_fwd_kernel<bf16_t>, dim3(grid_for(total)), dim3(256), 0, (hipStream_t)stream,
                           (const bf16_t *)gi, (const bf16_t *)gh, b_ih, b_hh, (const bf16_t *)h_prev, (bf16_t *)h_new,
                           (bf16_t *)saved, total, H);
    else
        hipLaunchKernelGGL(gru_gates_fwd_kernel<float>, dim3(grid_for(total)), dim3(256), 0, (hipStream_t)stream,
                           (const float *)gi, (const float *)gh, b_ih, b_hh, (const float *)h_prev, (float *)h_new,
                           (float *)saved, total, H);
    return check_launch();
}

int nsk_gru_gates_bwd(int dtype, int N, int H, const void *saved, const void *h_prev, const void *dh_a, const void *dh_b,
                      const void *dh_c, void *dgi, void *dgh, void *dh_direct, void *stream)
{
    if (N <= 0 || H <= 0 || !dtype_ok(dtype)) return NSK_ERR_BAD_DESC;
    if (!saved || !h_prev || !dh_a || !dgi || !dgh || !dh_direct) return NSK_ERR_NULL;
    if (unaligned16(saved) || unaligned16(h_prev) || unaligned16(dh_a) || (dh_b && unaligned16(dh_b)) ||
        (dh_c && unaligned16(dh_c)) || unaligned16(dgi) || unaligned16(dgh) || unaligned16(dh_direct))
        return NSK_ERR_ALIGNMENT;
    const long total = (long)N * H;
    if (dtype == NSK_BF16)
        hipLaunchKernelGGL(gru_gates_bwd_kernel<bf16_t>, dim3(grid_for(total)), dim3(256), 0, (hipStream_t)stream,
                           (const bf16_t *)saved, (const bf16_t *)h_prev, (const bf16_t *)dh_a, (const bf16_t *)dh_b,
                           (const bf16_t *)dh_c, (bf16_t *)dgi, (bf16_t *)dgh, (bf16_t *)dh_direct, total, H);
    else
        hipLaunchKernelGGL(gru_gates_bwd_kernel<float>, dim3(grid_for(total)), dim3(256), 0, (hipStream_t)stream,
                           (const float *)saved, (const float *)h_prev, (const float *)dh_a, (const float *)dh_b,
                           (const float *)dh_c, (float *)dgi, (float *)dgh, (float *)dh_direct, total, H);
    return check_launch();
}

int nsk_gru_step_supported(int N, int H) { return N > 0 && N <= 256 && H > 0 && H % 4 == 0; }

int nsk_gru_step_fwd(int dtype, int N, int H, const void *gi, const void *w_hh, const float *b_ih, const float *b_hh,
                     const void *h_prev, void *h_new, void *saved, void *stream)
{
    if (N <= 0 || H <= 0 || !dtype_ok(dtype)) return NSK_ERR_BAD_DESC;
    if (!gi || !w_hh || !b_ih || !b_hh || !h_prev || !h_new || !saved) return NSK_ERR_NULL;
    if (unaligned16(gi) || unaligned16(w_hh) || unaligned16(b_ih) || unaligned16(b_hh) || unaligned16(h_prev) ||
        unaligned16(h_new) || unaligned16(saved))
        return NSK_ERR_ALIGNMENT;
    if (!nsk_gru_step_supported(N, H)) return NSK_ERR_UNSUPPORTED;
    if (dtype == NSK_BF16)
        hipLaunchKernelGGL(gru_step_fwd_kernel<bf16_t>, dim3(H, (N + GS_THREADS / GS_LF - 1) / (GS_THREADS / GS_LF)), dim3(GS_THREADS), 0, (hipStream_t)stream, (const bf16_t *)gi,
                           (const bf16_t *)w_hh, b_ih, b_hh, (const bf16_t *)h_prev, (bf16_t *)h_new, (bf16_t *)saved, N, H);
    else
        hipLaunchKernelGGL(gru_step_fwd_kernel<float>, dim3(H, (N + GS_THREADS / GS_LF - 1) / (GS_THREADS / GS_LF)), dim3(GS_THREADS), 0, (hipStream_t)stream, (const float *)gi,
                           (const float *)w_hh, b_ih, b_hh, (const float *)h_prev, (float *)h_new, (float *)saved, N, H);
    return check_launch();
}

int nsk_gru_step_bwd(int dtype, int N, int H, const void *saved, const void *h_prev, const void *dh_a,
                     const void *dh_direct_next, const void *dgh_next, const void *w_hh_t, void *dgi, void *dgh,
                     void *dh_direct, void *stream)
{
    if (N <= 0 || H <= 0 || !dtype_ok(dtype)) return NSK_ERR_BAD_DESC;
    if (!saved || !h_prev || !w_hh_t || !dgi || !dgh || !dh_direct) return NSK_ERR_NULL;
    if (!dh_a && !dh_direct_next && !dgh_next) return NSK_ERR_NULL;   // no gradient at all
    if (unaligned16(saved) || unaligned16(h_prev) || (dh_a && unaligned16(dh_a)) ||
        (dh_direct_next && unaligned16(dh_direct_next)) || (dgh_next && unaligned16(dgh_next)) || unaligned16(w_hh_t) ||
        unaligned16(dgi) || unaligned16(dgh) || unaligned16(dh_direct))
        return NSK_ERR_ALIGNMENT;
    if (!nsk_gru_step_supported(N, H)) return NSK_ERR_UNSUPPORTED;
    if (dtype == NSK_BF16)
        hipLaunchKernelGGL(gru_step_bwd_kernel<bf16_t>, dim3(H, (N + GS_THREADS / GS_LB - 1) / (GS_THREADS / GS_LB)), dim3(GS_THREADS), 0, (hipStream_t)stream, (const bf16_t *)saved,
                           (const bf16_t *)h_prev, (const bf16_t *)dh_a, (const bf16_t *)dh_direct_next, (const bf16_t *)dgh_next,
                           (const bf16_t *)w_hh_t, (bf16_t *)dgi, (bf16_t *)dgh, (bf16_t *)dh_direct, N, H);
    else
        hipLaunchKernelGGL(gru_step_bwd_kernel<float>, dim3(H, (N + GS_THREADS / GS_LB - 1) / (GS_THREADS / GS_LB)), dim3(GS_THREADS), 0, (hipStream_t)stream, (const float *)saved,
                           (const float *)h_prev, (const float *)dh_a, (const float *)dh_direct_next, (const float *)dgh_next,
                           (const float *)w_hh_t, (float *)dgi, (float *)dgh, (float *)dh_direct, N, H);
    return check_launch();
}

}  // extern "C"

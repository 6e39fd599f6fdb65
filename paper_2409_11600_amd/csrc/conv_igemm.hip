// Implicit-GEMM convolution on the MFMA units of gfx950: the kernel behind conv forward and
// backward-data (both are "gather a shifted activation tile, multiply by a packed filter").
//
// GEMM view (the forward pass of a convolution layer of the ResNet recipe the paper trains,
// section "Experiments and Discussion"): rows m = output pixels, columns n = output channels,
// reduction k = (filter tap, input channel).  In NHWC each tap is a contiguous run of channels,
// so a k-tile is fetched with 16-byte loads and no im2col buffer ever exists in memory.
//
// Work decomposition: 256 threads = 4 wavefronts per block, block tile BM x BN, k-tile of 64
// bytes per row.  Tiles are staged through LDS (rows padded to 80 bytes so the 16-byte fragment
// reads of 8 consecutive lanes cover all 32 banks once) with register prefetch of the next
// k-tile and two LDS buffers, so one barrier per k-tile suffices.  Each wavefront owns a
// WM x WN sub-tile made of 32x32 MFMA accumulators.
#include <stdlib.h>

#include "nsk_internal.h"

namespace nsk {
namespace {

// BKB = bytes of reduction index per k-tile row (64 or 128); LDS rows are padded by 16 bytes so
// that the 16-byte fragment reads of 8 consecutive rows fall into 8 different bank groups.
template <typename T> struct Traits;
template <> struct Traits<float> {
    static constexpr int VEC = 4;
    typedef f32x4 Vec;
};
template <> struct Traits<bf16_t> {
    static constexpr int VEC = 8;
    typedef bf16x8 Vec;
};

template <typename Vec> __device__ inline Vec zero_vec()
{
    Vec v;
#pragma unroll
    for (int i = 0; i < (int)(sizeof(Vec) / sizeof(v[0])); ++i) v[i] = 0;
    return v;
}

__device__ inline float to_float(float v) { return v; }
__device__ inline float to_float(bf16_t v) { return (float)v; }

template <typename T, int BM, int BN, int WM, int WN, int BKB, bool VECLOAD>
__global__ __launch_bounds__(256) void igemm_kernel(const IgemmArgs a)
{
    typedef Traits<T> TR;
    typedef typename TR::Vec Vec;
    constexpr int VEC = TR::VEC, BK = BKB / (int)sizeof(T), LDK = BK + VEC;
    constexpr int WAVES_N = BN / WN;
    static_assert((BM / WM) * WAVES_N == 4, "four wavefronts per block");
    constexpr int FM = WM / 32, FN = WN / 32;
    constexpr int VPR = BK / VEC;        // 16-byte vectors per tile row
    constexpr int RPP = 256 / VPR;       // tile rows loaded per pass of the 256 threads
    constexpr int A_PASSES = BM / RPP;
    constexpr int B_PASSES = (BN + RPP - 1) / RPP;

    __shared__ __attribute__((aligned(16))) T smem_ab[2 * (BM + BN) * LDK];
    T(*As)[BM * LDK] = (T(*)[BM * LDK])smem_ab;
    T(*Bs)[BN * LDK] = (T(*)[BN * LDK])(smem_ab + 2 * BM * LDK);
    __shared__ long out_off[BM];
    __shared__ short s_offh[kMaxTaps], s_offw[kMaxTaps];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int m0 = blockIdx.x * BM;
    const int n0 = blockIdx.y * BN;
    // grouped convolution: blockIdx.z names the group (0 for a plain launch); ld = channels between two source pixels
    const int grp = blockIdx.z, ld = a.src_ld;
    const int src_c0 = grp * a.Cs;            // first source channel of the group
    const long wrow0 = (long)grp * a.Ngemm;   // first filter row = first output channel of the group

    if (tid < kMaxTaps) {
        s_offh[tid] = a.off_h[tid];
        s_offw[tid] = a.off_w[tid];
    }

    const T *__restrict__ src = (const T *)a.src;
    const T *__restrict__ wpk = (const T *)a.wpk;

    // Each thread gathers the same rows in every k-tile: decode them once.  For the vector path the
    // per-row state is a 32-bit byte offset of the row's base pixel and a bit mask of the taps that
    // fall inside the image; a k-tile then costs one shift, one add and one select per load.  Loads go
    // through buffer descriptors: an offset of ~0 is out of range and returns zeros without a branch.
    const int kv = tid % VPR;  // which 16-byte vector of the k-tile row
    const int r0 = tid / VPR;  // row within a pass of RPP rows
    int a_img[A_PASSES], a_bh[A_PASSES], a_bw[A_PASSES];
    bool a_ok[A_PASSES];
    unsigned a_base[A_PASSES];
    unsigned long long a_mask[A_PASSES];
#pragma unroll
    for (int u = 0; u < A_PASSES; ++u) {
        const int row = r0 + RPP * u;
        const int m = m0 + row;
        a_ok[u] = m < a.M;
        const int mm = a_ok[u] ? m : 0;
        const int per_img = a.Mi * a.Mj;
        const int img = mm / per_img;
        const int rem = mm - img * per_img;
        const int i = rem / a.Mj;
        const int j = rem - i * a.Mj;
        a_img[u] = img * a.Hs;
        a_bh[u] = i * a.mult_h + a.add_h;
        a_bw[u] = j * a.mult_w + a.add_w;
        a_base[u] = (unsigned)(((((long)a_img[u] + a_bh[u]) * a.Ws + a_bw[u]) * ld + src_c0) * (long)sizeof(T));
        if (kv == 0)
            out_off[row] = a_ok[u] ? (((long)img * a.Ho + (i * a.osh + a.oa)) * a.Wo + (j * a.osw + a.ob)) * a.Co + wrow0
                                   : -1L;
    }
    __syncthreads();
    if (VECLOAD) {
#pragma unroll
        for (int u = 0; u < A_PASSES; ++u) {
            unsigned long long mask = 0;
            if (a_ok[u])
                for (int t = 0; t < a.ntaps; ++t) {
                    const int h = a_bh[u] + s_offh[t], w = a_bw[u] + s_offw[t];
                    if ((unsigned)h < (unsigned)a.Hs && (unsigned)w < (unsigned)a.Ws) mask |= 1ull << t;
                }
            a_mask[u] = mask;
        }
    }
    const __amdgpu_buffer_rsrc_t src_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.src, 0, a.src_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t wpk_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.wpk, 0, a.wpk_bytes, 0x00020000);

    Vec ra[A_PASSES], rb[B_PASSES];
    int cur_tap = 0, cur_c = kv * VEC;  // position of this thread's vector inside (tap, channel)
    if (VECLOAD) {
        while (cur_c >= a.Cs && cur_tap < a.ntaps) {
            cur_c -= a.Cs;
            ++cur_tap;
        }
    }
    unsigned b_row_off[B_PASSES];
#pragma unroll
    for (int u = 0; u < B_PASSES; ++u) {
        const int row = r0 + RPP * u;
        const int n = n0 + row;
        b_row_off[u] = (row < BN && n < a.Ngemm) ? (unsigned)((wrow0 + n) * a.Ktot * (long)sizeof(T)) : ~0u;
    }

    auto load_tile = [&](int kt) {
        const int kk = kt * BK + kv * VEC;
        if (VECLOAD) {
            const bool kok = kk < a.Ktot;
            const int tap = kok ? cur_tap : 0;
            const unsigned delta = (unsigned)((((int)s_offh[tap] * a.Ws + (int)s_offw[tap]) * ld + cur_c) * (int)sizeof(T));
#pragma unroll
            for (int u = 0; u < A_PASSES; ++u) {
                const bool ok = kok && ((a_mask[u] >> tap) & 1ull);
                const unsigned off = ok ? a_base[u] + delta : ~0u;
                ra[u] = __builtin_bit_cast(Vec, __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, off, 0, 0));
            }
#pragma unroll
            for (int u = 0; u < B_PASSES; ++u) {
                const unsigned off = (kok && b_row_off[u] != ~0u) ? b_row_off[u] + (unsigned)(kk * (int)sizeof(T)) : ~0u;
                rb[u] = __builtin_bit_cast(Vec, __builtin_amdgcn_raw_buffer_load_b128(wpk_rsrc, off, 0, 0));
            }
            // advance to the next k-tile
            cur_c += BK;
            while (cur_c >= a.Cs && cur_tap < a.ntaps) {
                cur_c -= a.Cs;
                ++cur_tap;
            }
        } else {
            // Element-wise gather for channel counts that are not a multiple of the vector width
            // (the 3-channel image stem).
#pragma unroll
            for (int u = 0; u < A_PASSES; ++u) ra[u] = zero_vec<Vec>();
#pragma unroll
            for (int u = 0; u < B_PASSES; ++u) rb[u] = zero_vec<Vec>();
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const int k = kk + e;
                if (k < a.Ktot) {
                    const int tap = k / a.Cs;
                    const int c = k - tap * a.Cs;
                    const int oh = s_offh[tap], ow = s_offw[tap];
#pragma unroll
                    for (int u = 0; u < A_PASSES; ++u) {
                        const int h = a_bh[u] + oh, w = a_bw[u] + ow;
                        const bool ok = a_ok[u] && (unsigned)h < (unsigned)a.Hs && (unsigned)w < (unsigned)a.Ws;
                        if (ok) ra[u][e] = src[((long)(a_img[u] + h) * a.Ws + w) * ld + src_c0 + c];
                    }
#pragma unroll
                    for (int u = 0; u < B_PASSES; ++u) {
                        const int row = r0 + RPP * u;
                        const int n = n0 + row;
                        if (row < BN && n < a.Ngemm) rb[u][e] = wpk[(wrow0 + n) * a.Ktot + k];
                    }
                }
            }
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int u = 0; u < A_PASSES; ++u) *(Vec *)&As[buf][(r0 + RPP * u) * LDK + kv * VEC] = ra[u];
#pragma unroll
        for (int u = 0; u < B_PASSES; ++u) {
            const int row = r0 + RPP * u;
            if (row < BN) *(Vec *)&Bs[buf][row * LDK + kv * VEC] = rb[u];
        }
    };

    // The filter rows are the MFMA "A" operand and the pixels the "B" operand, so a lane ends up with 4
    // CONSECUTIVE CHANNELS of one pixel per accumulator quad: acc[mi][ni][4g+j] is channel
    // 32*ni + 8*g + 4*(lane/32) + j of pixel 32*mi + lane%32 of the wavefront's sub-tile.
    const int frow = lane & 31, fk = lane >> 5;
    T *__restrict__ out = (T *)a.out;
    const int wcol0 = n0 + wn * WN;   // first output channel of this wavefront
    f32x16 acc[FM][FN];
#pragma unroll
    for (int mi = 0; mi < FM; ++mi)
#pragma unroll
        for (int ni = 0; ni < FN; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;
    if (a.accumulate && a.vec_out) {
        // start from the old values: the sum is then rounded to the storage type exactly once
#pragma unroll
        for (int mi = 0; mi < FM; ++mi) {
            const long off = out_off[wm * WM + mi * 32 + frow];
#pragma unroll
            for (int ni = 0; ni < FN; ++ni)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int col = wcol0 + ni * 32 + g * 8 + fk * 4;
                    if (off >= 0 && col < a.Ngemm) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc[mi][ni][g * 4 + j] = to_float(out[off + col + j]);
                    }
                }
        }
    }

    const int nk = (a.Ktot + BK - 1) / BK;
    if (nk > 0) {
        load_tile(0);
        store_tile(0);
    }
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_tile(kt + 1);
        const T *pa = &As[buf][(wm * WM + frow) * LDK + fk * VEC];
        const T *pb = &Bs[buf][(wn * WN + frow) * LDK + fk * VEC];
#pragma unroll
        for (int ks = 0; ks < BK; ks += 2 * VEC) {
            Vec af[FM], bfv[FN];
#pragma unroll
            for (int mi = 0; mi < FM; ++mi) af[mi] = *(const Vec *)(pa + mi * 32 * LDK + ks);
#pragma unroll
            for (int ni = 0; ni < FN; ++ni) bfv[ni] = *(const Vec *)(pb + ni * 32 * LDK + ks);
            if constexpr (sizeof(T) == 2) {
#pragma unroll
                for (int mi = 0; mi < FM; ++mi)
#pragma unroll
                    for (int ni = 0; ni < FN; ++ni)
                        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfv[ni], af[mi], acc[mi][ni], 0, 0, 0);
            } else {
                // Lane (row, half) holds k = 4*half + t of this group of 8; the same map is used
                // for both operands, so the four steps together cover the 8 k exactly once.
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int mi = 0; mi < FM; ++mi)
#pragma unroll
                        for (int ni = 0; ni < FN; ++ni)
                            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(bfv[ni][t], af[mi][t], acc[mi][ni], 0, 0, 0);
            }
        }
        if (kt + 1 < nk) store_tile(buf ^ 1);
        __syncthreads();
    }

    if (a.vec_out) {
        // Round to the storage type, transpose one 32 x 32 accumulator tile at a time through this
        // wavefront's strip of the (now idle) operand buffers, and store 16 contiguous bytes per lane.
        typedef T T4 __attribute__((ext_vector_type(4)));
        constexpr int SROW = 32 * (int)sizeof(T) + 16;      // staged bytes per pixel (padded)
        constexpr int CPP = 32 * (int)sizeof(T) / 16;       // 16-byte chunks per pixel
        static_assert(4 * 32 * SROW <= (int)sizeof(smem_ab), "epilogue staging fits in the operand buffers");
        unsigned char *my_st = (unsigned char *)smem_ab + wave * (32 * SROW);
        // Statistics epilogue (forward with a batch-norm behind it): a lane always reads back the same 16-byte piece
        // (VEC channels) of each staged row, so it adds those channels up over all the rows it stores; one cross-lane
        // reduction per block and one row of partial sums per wavefront.
        float ssum[FN][VEC], ssq[FN][VEC];
#pragma unroll
        for (int ni = 0; ni < FN; ++ni)
#pragma unroll
            for (int e = 0; e < VEC; ++e) ssum[ni][e] = ssq[ni][e] = 0.f;
#pragma unroll
        for (int mi = 0; mi < FM; ++mi)
#pragma unroll
            for (int ni = 0; ni < FN; ++ni) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    T4 pk;
#pragma unroll
                    for (int j = 0; j < 4; ++j) pk[j] = (T)acc[mi][ni][g * 4 + j];
                    *(T4 *)(my_st + frow * SROW + (g * 8 + fk * 4) * (int)sizeof(T)) = pk;
                }
#pragma unroll
                for (int jj = 0; jj < 32 * CPP / 64; ++jj) {
                    const int idx = lane + 64 * jj, pos = idx / CPP, ck = idx % CPP;
                    const Vec v = *(const Vec *)(my_st + pos * SROW + ck * 16);
                    const long off = out_off[wm * WM + mi * 32 + pos];
                    const int col = wcol0 + ni * 32 + ck * VEC;
                    if (off >= 0 && col < a.Ngemm) {
                        *(Vec *)(out + off + col) = v;
                        if (a.stats) {
#pragma unroll
                            for (int e = 0; e < VEC; ++e) {
                                const float f = to_float(v[e]);
                                ssum[ni][e] += f;
                                ssq[ni][e] += f * f;
                            }
                        }
                    }
                }
            }
        if (a.stats) {
            const int row = blockIdx.x * (BM / WM) + wm, ck = lane % CPP;
#pragma unroll
            for (int ni = 0; ni < FN; ++ni) {
#pragma unroll
                for (int e = 0; e < VEC; ++e)
#pragma unroll
                    for (int o = CPP; o < 64; o <<= 1) {
                        ssum[ni][e] += __shfl_xor(ssum[ni][e], o, 64);
                        ssq[ni][e] += __shfl_xor(ssq[ni][e], o, 64);
                    }
                const int col = wcol0 + ni * 32 + ck * VEC;
                if (lane < CPP && col < a.Ngemm) {
                    // 16-byte stores: a handful of lanes writing single floats would cost one memory instruction each
                    float *r0 = a.stats + (size_t)row * a.Ngemm + col;
                    float *r1 = r0 + (size_t)a.stats_rows * a.Ngemm;
#pragma unroll
                    for (int e = 0; e < VEC; e += 4) {
                        *(f32x4 *)(r0 + e) = f32x4{ssum[ni][e], ssum[ni][e + 1], ssum[ni][e + 2], ssum[ni][e + 3]};
                        *(f32x4 *)(r1 + e) = f32x4{ssq[ni][e], ssq[ni][e + 1], ssq[ni][e + 2], ssq[ni][e + 3]};
                    }
                }
            }
        }
    } else {
        // element-wise stores (output rows that are not 16-byte granular)
#pragma unroll
        for (int mi = 0; mi < FM; ++mi) {
            const long off = out_off[wm * WM + mi * 32 + frow];
            if (off < 0) continue;
#pragma unroll
            for (int ni = 0; ni < FN; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int col = wcol0 + ni * 32 + 8 * (v >> 2) + 4 * fk + (v & 3);
                    if (col < a.Ngemm) {
                        float r = acc[mi][ni][v];
                        if (a.accumulate) r += to_float(out[off + col]);
                        out[off + col] = (T)r;
                    }
                }
        }
    }
}

template <typename T, int BM, int BN, int WM, int WN, int BKB>
int launch_tile(const IgemmArgs &a, bool vec, hipStream_t stream)
{
    dim3 grid(ceil_div(a.M, BM), ceil_div(a.Ngemm, BN), a.groups);
    if (vec)
        hipLaunchKernelGGL((igemm_kernel<T, BM, BN, WM, WN, BKB, true>), grid, dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL((igemm_kernel<T, BM, BN, WM, WN, 64, false>), grid, dim3(256), 0, stream, a);
    return check_launch();
}

// NSK_IGEMM_TILE=<n> forces a tile variant (A/B experiments); unset or 0 = automatic choice.
int forced_tile()
{
    return hooks().igemm_tile;
}

// Automatic tile choice: 0 = 256x32 (64-row wavefront tiles), 1 = 128x64 (32-row), 2 = 128x128 (64-row).
int auto_tile(const IgemmArgs &a, int es)
{
    if (a.Ngemm <= 32) return 0;
    if (a.Ngemm <= 64) return 1;
    if ((long)a.Ktot * es >= 1024) return 2;
    return 1;
}

template <typename T> int launch_typed(const IgemmArgs &a, hipStream_t stream)
{
    constexpr int VEC = Traits<T>::VEC;
    // (for a grouped launch Cs % VEC == 0 also puts every group's channel run and filter rows on 16-byte boundaries)
    const bool vec = a.Cs % VEC == 0 && a.src_ld % VEC == 0 && a.Ktot % VEC == 0 && ((uintptr_t)a.src % 16 == 0) &&
                     ((uintptr_t)a.wpk % 16 == 0);
    switch (forced_tile()) {
    case 1: return launch_tile<T, 256, 64, 64, 64, 64>(a, vec, stream);
    case 2: return launch_tile<T, 256, 64, 64, 64, 128>(a, vec, stream);
    case 3: return launch_tile<T, 128, 64, 32, 64, 64>(a, vec, stream);
    case 4: return launch_tile<T, 128, 64, 32, 64, 128>(a, vec, stream);
    case 5: return launch_tile<T, 128, 128, 64, 64, 64>(a, vec, stream);
    case 6: return launch_tile<T, 128, 128, 64, 64, 128>(a, vec, stream);
    default: break;
    }
    // Measured on MI355X: with 64 or fewer columns the 128-row tile wins (more blocks in flight hide
    // the per-block prologue and epilogue); wide problems with a long reduction take 128x128 tiles
    // with 128-byte k-tiles (half as many barriers).
    switch (auto_tile(a, (int)sizeof(T))) {
    case 0: return launch_tile<T, 256, 32, 64, 32, 64>(a, vec, stream);
    case 1: return launch_tile<T, 128, 64, 32, 64, 64>(a, vec, stream);
    default: return launch_tile<T, 128, 128, 64, 64, 128>(a, vec, stream);
    }
}

}  // namespace

int igemm_stats_rows(int dtype, const IgemmArgs &a)
{
    // the same order of tests as launch_igemm
    if (a.M <= 0 || a.Ngemm <= 0 || a.accumulate) return 0;
    if (forced_tile() != 0 || a.groups > 1) return 0;
    if (tiny_src_applicable(dtype, a) || tiny_out_applicable(dtype, a)) return 0;   // no statistics epilogue there
    if (halo64_applicable(dtype, a)) return halo64_stats_rows(a);
    if (halo64_f32_applicable(dtype, a)) return halo64_f32_stats_rows(a);
    if (fs64_fwd_s2_applicable(dtype, a)) return fs64_fwd_s2_stats_rows(a);
    if (conv_pw_applicable(dtype, a)) return conv_pw_stats_rows(a);
    if (halo_wide_applicable(dtype, a)) return halo_wide_stats_rows(a);
    if (halo_wide_fwd_s2_applicable(dtype, a)) return halo_wide_fwd_s2_stats_rows(a);
    if (igemm_big_applicable(dtype, a)) return igemm_big_stats_rows(a);
    // generic kernel: needs the vector epilogue; one row per wavefront row of every row block.  Measured: with a
    // short reduction the per-block cross-lane sums and the many rows of partial sums cost more than the separate
    // statistics pass they replace (config 5 stage A: +45 us on a 140 us layer), so only long reductions use it.
    const int vec = dtype == NSK_BF16 ? 8 : 4;
    if (!(a.Ngemm % vec == 0 && a.Co % vec == 0 && (uintptr_t)a.out % 16 == 0)) return 0;
    if (a.Ktot < 1024 && !hooks().stats_always) return 0;   // the variable is a test hook
    if (a.Ngemm % 4 != 0) return 0;   // 16-byte stores of the partial sums
    static const int bm[3] = {256, 128, 128}, wm[3] = {64, 32, 64};
    const int t = auto_tile(a, dtype == NSK_BF16 ? 2 : 4);
    return ceil_div(a.M, bm[t]) * (bm[t] / wm[t]);
}

bool igemm_act_fused(int dtype, const IgemmArgs &a)
{
    // the same order of tests as launch_igemm, up to the kernels that have the fused load
    if (a.M <= 0 || a.Ngemm <= 0 || a.accumulate || a.groups > 1 || a.zero_cell || forced_tile() != 0) return false;
    if (tiny_src_applicable(dtype, a) || tiny_out_applicable(dtype, a) || halo64_applicable(dtype, a)) return false;
    return halo64_f32_applicable(dtype, a);
}

int launch_igemm(int dtype, const IgemmArgs &a, hipStream_t stream)
{
    if (a.M <= 0 || a.Ngemm <= 0) return NSK_OK;
    if (a.act && !igemm_act_fused(dtype, a)) return NSK_ERR_BAD_DESC;   // the caller applies the activation itself
    const bool grouped = a.groups > 1;   // only the generic kernel knows about groups
    if (grouped && (a.groups > 65535 || a.src_ld != a.groups * a.Cs || a.zero_cell || a.stats)) return NSK_ERR_BAD_DESC;
    if (a.zero_cell) return launch_conv_pw(a, stream);   // the caller has checked that this kernel applies
    const bool special = forced_tile() == 0 && !grouped;
    if (special && tiny_src_applicable(dtype, a)) return launch_tiny_src(dtype, a, stream);
    if (special && tiny_out_applicable(dtype, a)) return launch_tiny_out(dtype, a, stream);
    if (special && halo64_applicable(dtype, a)) return launch_halo64(a, stream);
    if (special && halo64_f32_applicable(dtype, a)) return launch_halo64_f32(a, stream);
    if (special && fs64_fwd_s2_applicable(dtype, a)) return launch_fs64_fwd_s2(a, stream);
    if (special && conv_pw_applicable(dtype, a)) return launch_conv_pw(a, stream);
    if (special && halo_wide_applicable(dtype, a)) return launch_halo_wide(a, stream);
    if (special && halo_wide_fwd_s2_applicable(dtype, a)) return launch_halo_wide_fwd_s2(a, stream);
    if (special && igemm_big_applicable(dtype, a)) return launch_igemm_big(a, stream);
    if (grouped && forced_tile() == 0 && !hooks().no_depthwise && depthwise_applicable(dtype, a))
        return launch_depthwise(dtype, a, stream);
    IgemmArgs b = a;
    if (!grouped) {
        b.groups = 1;
        b.src_ld = b.Cs;
    }
    const int vec = dtype == NSK_BF16 ? 8 : 4;
    b.vec_out = (b.Ngemm % vec == 0 && b.Co % vec == 0 && (uintptr_t)b.out % 16 == 0) ? 1 : 0;
    return dtype == NSK_BF16 ? launch_typed<bf16_t>(b, stream) : launch_typed<float>(b, stream);
}

}  // namespace nsk

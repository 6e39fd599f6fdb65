// Short-reduction convolution for narrow bf16 layers: one, two or four taps and at most 256 reduction indices in
// all (plus the nine taps of a strided 3x3 layer on 64 -> 64 channels).  These are the 1x1 layers of a bottleneck block (forward with any stride, and their backward-data pass) and
// the residue classes of the backward-data pass of a stride-2 3x3 layer on 64 channels, on the large early feature
// maps of the ResNet recipe the paper trains (section "Experiments and Discussion").
//
// Such layers move about ten times more bytes per multiply than the matrix units need, so the kernel is built
// around the memory stream and not around the multiply:
//   * the whole filter ([Ngemm][Cs], at most 64 KB) is copied to LDS once per block and stays there;
//   * a wavefront owns a tile of 32*FM pixels and loads their channels straight into registers in the MFMA
//     operand layout (lane = pixel, 16 bytes = 8 consecutive channels): the activations never pass through LDS;
//   * the loads of the next tile are issued before the current tile is multiplied, so every wavefront keeps a
//     whole tile of loads in flight while it multiplies, converts and stores;
//   * wavefronts never wait for each other after the filter copy (no barrier in the tile loop);
//   * output rows are staged through a per-wavefront LDS strip so that 8 lanes store 128 contiguous bytes;
//   * an accumulating launch fetches the old output values the same way, one 64-channel chunk ahead, and adds them
//     to the fp32 sums before the single rounding.
// One block of 4 wavefronts per CU (the register file then allows two tiles of up to 256 channels per lane).
#include <stdlib.h>

#include "nsk_internal.h"

namespace nsk {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kPwGrid = 256;            // blocks; fixed so that the number of statistics rows is a shape property
constexpr unsigned PW_OOB = 0xF0000000u;  // beyond every buffer: loads return zero, stores are dropped
constexpr int PW_SROW = 64 * 2 + 16;    // staged bytes per pixel: 64 channels and a 16-byte pad
constexpr int PW_SROW_F32 = 64 * 4 + 16;   // the same for fp32 sums (accumulating launches)
constexpr int PW_MAX_NCH = 4;           // column chunks of 64 (Ngemm <= 256)

struct PwArgs {
    IgemmArgs g;
    int tiles;
    int zero_cell;   // also write zeros to the other pixels of each row's 2x2 output cell (see IgemmArgs::zero_cell)
    unsigned out_bytes;
    unsigned long long magic_img, magic_row;   // ceil(2^40 / (Mi*Mj)), ceil(2^40 / Mj)
};

template <int KS, int FM, int TAPS, bool ACC>
__global__ __launch_bounds__(256, 1) void conv_pw_kernel(const PwArgs pa)
{
    const IgemmArgs &a = pa.g;
    constexpr int TM = 32 * FM;                      // pixels per wavefront tile
    constexpr int RPL = (TM + 63) / 64;              // tile rows decoded per lane
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int KPT = KS / TAPS;                   // k-steps (16 channels) per tap
    constexpr int STRIP = ACC ? 32 * PW_SROW_F32 : 32 * PW_SROW;   // bytes of the transposing strip
    const int Cs = 16 * KPT;
    const int WROW = KS * 32 + 16;                   // filter row pitch: 16 bytes of padding spread the rows over the banks
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int frow = lane & 31, fk = lane >> 5;
    unsigned char *w_lds = smem;
    unsigned char *my_st = smem + (size_t)a.Ngemm * WROW + wave * (STRIP + (2 * TAPS + 2) * TM * 4);
    unsigned *soff_lds = (unsigned *)(my_st + STRIP);   // [2][TAPS][TM] byte offsets of the tile's source pixels
    unsigned *ooff_lds = soff_lds + 2 * TAPS * TM;             // [2][TM] byte offsets of its output pixels (+ flags)

    const __amdgpu_buffer_rsrc_t src_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.src, 0, a.src_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t wpk_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.wpk, 0, a.wpk_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t out_rsrc = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, pa.out_bytes, 0x00020000);

    // filter -> LDS
    for (int idx = tid; idx < a.Ngemm * (2 * KS); idx += 256) {
        const int n = idx / (2 * KS), ch = idx % (2 * KS);
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(wpk_rsrc, (unsigned)((n * KS * 16 + ch * 8) * 2), 0, 0);
        *(u32x4 *)(w_lds + n * WROW + ch * 16) = v;
    }
    __syncthreads();

    const int per_img = a.Mi * a.Mj;
    // Source (per tap) and output byte offsets of the tile's pixels (PW_OOB for rows past the end and for source
    // positions outside the image), written to this wavefront's LDS arrays of the given parity.  Output offsets are
    // multiples of 16; their two low bits say whether the pixel to the right / below exists (zero_cell).
    auto decode = [&](int tile, int par) {
#pragma unroll
        for (int u = 0; u < RPL; ++u) {
            const int r = lane + 64 * u;
            const int m = tile * TM + r;
            unsigned so[TAPS], oo = PW_OOB;
#pragma unroll
            for (int tp = 0; tp < TAPS; ++tp) so[tp] = PW_OOB;
            if (r < TM && m < a.M) {
                const int img = (int)(((unsigned long long)m * pa.magic_img) >> 40);
                const int rem = m - img * per_img;
                const int i = (int)(((unsigned long long)rem * pa.magic_row) >> 40);
                const int j = rem - i * a.Mj;
#pragma unroll
                for (int tp = 0; tp < TAPS; ++tp) {
                    const int h = i * a.mult_h + a.add_h + a.off_h[tp], w = j * a.mult_w + a.add_w + a.off_w[tp];
                    if ((unsigned)h < (unsigned)a.Hs && (unsigned)w < (unsigned)a.Ws)
                        so[tp] = (unsigned)(((img * a.Hs + h) * a.Ws + w) * Cs) * 2u;
                }
                const int ho = i * a.osh + a.oa, wo = j * a.osw + a.ob;
                oo = (unsigned)(((img * a.Ho + ho) * a.Wo + wo) * a.Co) * 2u;
                oo |= (wo + 1 < a.Wo ? 1u : 0u) | (ho + 1 < a.Ho ? 2u : 0u);
            }
            if (r < TM) {
#pragma unroll
                for (int tp = 0; tp < TAPS; ++tp) soff_lds[(par * TAPS + tp) * TM + r] = so[tp];
                ooff_lds[par * TM + r] = oo;
            }
        }
    };
    auto issue = [&](u32x4 (&A)[FM][KS], int par) {
#pragma unroll
        for (int mi = 0; mi < FM; ++mi) {
#pragma unroll
            for (int tp = 0; tp < TAPS; ++tp) {
                const unsigned so = soff_lds[(par * TAPS + tp) * TM + 32 * mi + frow] + (unsigned)(fk * 16);
#pragma unroll
                for (int kk = 0; kk < KPT; ++kk)
                    A[mi][tp * KPT + kk] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, so + kk * 32, 0, 0);
            }
        }
    };

    // Accumulating launches: the old values of the 64-channel chunk a lane will store (same pixel, same 16 bytes),
    // fetched one chunk ahead of the multiply that needs them.
    u32x4 O[2][FM][4];
    auto issue_old = [&](u32x4 (&Ob)[FM][4], int par, int nc) {
#pragma unroll
        for (int mi = 0; mi < FM; ++mi)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const int idx = lane + 64 * jj, pos = idx >> 3, ck = idx & 7;
                const unsigned oo = ooff_lds[par * TM + 32 * mi + pos] & ~15u;
                Ob[mi][jj] = __builtin_amdgcn_raw_buffer_load_b128(out_rsrc, oo + (unsigned)((nc * 64 + ck * 8) * 2), 0, 0);
            }
    };

    float ssum[PW_MAX_NCH][8], ssq[PW_MAX_NCH][8];
#pragma unroll
    for (int nc = 0; nc < PW_MAX_NCH; ++nc)
#pragma unroll
        for (int e = 0; e < 8; ++e) ssum[nc][e] = ssq[nc][e] = 0.f;
    const int nch = a.Ngemm >> 6;
    const bool want_stats = a.stats != nullptr;

    auto compute = [&](const u32x4 (&A)[FM][KS], int par, bool has_next) {
#pragma unroll
        for (int nc = 0; nc < PW_MAX_NCH; ++nc) {
            if (nc >= nch) break;
            if constexpr (ACC) {
                if (nc + 1 < nch) issue_old(O[(nc + 1) & 1], par, nc + 1);
            }
            f32x16 acc[FM][2];
#pragma unroll
            for (int mi = 0; mi < FM; ++mi)
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;
            const unsigned char *wb = w_lds + (nc * 64 + frow) * WROW + fk * 16;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 b0 = *(const bf16x8 *)(wb + ks * 32);
                const bf16x8 b1 = *(const bf16x8 *)(wb + 32 * WROW + ks * 32);
#pragma unroll
                for (int mi = 0; mi < FM; ++mi) {
                    const bf16x8 av = __builtin_bit_cast(bf16x8, A[mi][ks]);
                    acc[mi][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b0, av, acc[mi][0], 0, 0, 0);
                    acc[mi][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b1, av, acc[mi][1], 0, 0, 0);
                }
            }
            // acc[mi][ni][4g+j] = channel 64nc + 32ni + 8g + 4fk + j of pixel 32mi + frow: round, transpose 32 pixels x 64
            // channels through the strip, store 128 bytes per pixel with 8 lanes.
#pragma unroll
            for (int mi = 0; mi < FM; ++mi) {
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        if constexpr (ACC) {
                            *(f32x4 *)(my_st + frow * PW_SROW_F32 + (ni * 32 + g * 8 + fk * 4) * 4) =
                                f32x4{acc[mi][ni][g * 4], acc[mi][ni][g * 4 + 1], acc[mi][ni][g * 4 + 2], acc[mi][ni][g * 4 + 3]};
                        } else {
                            bf16x4 pk;
#pragma unroll
                            for (int j = 0; j < 4; ++j) pk[j] = (bf16_t)acc[mi][ni][g * 4 + j];
                            *(bf16x4 *)(my_st + frow * PW_SROW + (ni * 32 + g * 8 + fk * 4) * 2) = pk;
                        }
                    }
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const int idx = lane + 64 * jj, pos = idx >> 3, ck = idx & 7;
                    u32x4 v;
                    if constexpr (ACC) {
                        // old value + sum of products, rounded to the storage type once
                        const f32x4 lo = *(const f32x4 *)(my_st + pos * PW_SROW_F32 + ck * 32);
                        const f32x4 hi = *(const f32x4 *)(my_st + pos * PW_SROW_F32 + ck * 32 + 16);
                        const bf16x8 old = __builtin_bit_cast(bf16x8, O[nc & 1][mi][jj]);
                        bf16x8 r;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            r[e] = (bf16_t)(lo[e] + (float)old[e]);
                            r[e + 4] = (bf16_t)(hi[e] + (float)old[e + 4]);
                        }
                        v = __builtin_bit_cast(u32x4, r);
                    } else {
                        v = *(const u32x4 *)(my_st + pos * PW_SROW + ck * 16);
                    }
                    const unsigned oraw = ooff_lds[par * TM + 32 * mi + pos];
                    const unsigned oo = oraw & ~15u, cb = (unsigned)((nc * 64 + ck * 8) * 2);
                    __builtin_amdgcn_raw_buffer_store_b128(v, out_rsrc, oo + cb, 0, 0);
                    if (!ACC && pa.zero_cell) {
                        const u32x4 z = {0u, 0u, 0u, 0u};
                        const unsigned right = (unsigned)(a.Co * 2), below = (unsigned)(a.Wo * a.Co * 2);
                        __builtin_amdgcn_raw_buffer_store_b128(z, out_rsrc, (oraw & 1u) ? oo + right + cb : PW_OOB, 0, 0);
                        __builtin_amdgcn_raw_buffer_store_b128(z, out_rsrc, (oraw & 2u) ? oo + below + cb : PW_OOB, 0, 0);
                        __builtin_amdgcn_raw_buffer_store_b128(z, out_rsrc, (oraw & 3u) == 3u ? oo + below + right + cb : PW_OOB, 0, 0);
                    }
                    if (!ACC && want_stats && oo != PW_OOB) {
                        const bf16x8 bv = __builtin_bit_cast(bf16x8, v);
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const float f = (float)bv[e];
                            ssum[nc][e] += f;
                            ssq[nc][e] += f * f;
                        }
                    }
                }
            }
        }
        if constexpr (ACC) {
            if (has_next) issue_old(O[0], par ^ 1, 0);   // first chunk of the next tile (its offsets are decoded already)
        }
    };

    u32x4 A0[FM][KS], A1[FM][KS];
    const int stride = gridDim.x * 4;
    int t = blockIdx.x * 4 + wave;
    if (t < pa.tiles) {
        decode(t, 0);
        if constexpr (ACC) issue_old(O[0], 0, 0);
        issue(A0, 0);
    }
    while (t < pa.tiles) {
        bool has_next = t + stride < pa.tiles;
        if (has_next) {
            decode(t + stride, 1);
            issue(A1, 1);
        }
        __builtin_amdgcn_sched_barrier(0);
        compute(A0, 0, has_next);
        __builtin_amdgcn_sched_barrier(0);
        t += stride;
        if (t >= pa.tiles) break;
        has_next = t + stride < pa.tiles;
        if (has_next) {
            decode(t + stride, 0);
            issue(A0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        compute(A1, 1, has_next);
        __builtin_amdgcn_sched_barrier(0);
        t += stride;
    }

    if (!ACC && want_stats) {
        // lanes with equal (lane & 7) hold the same channels: add them up, one row of partial sums per wavefront
        const int row = blockIdx.x * 4 + wave, ck = lane & 7;
#pragma unroll
        for (int nc = 0; nc < PW_MAX_NCH; ++nc) {
            if (nc >= nch) break;
#pragma unroll
            for (int e = 0; e < 8; ++e)
#pragma unroll
                for (int o = 8; o < 64; o <<= 1) {
                    ssum[nc][e] += __shfl_xor(ssum[nc][e], o, 64);
                    ssq[nc][e] += __shfl_xor(ssq[nc][e], o, 64);
                }
            if (lane < 8) {
                float *r0 = a.stats + (size_t)row * a.Ngemm + nc * 64 + ck * 8;
                float *r1 = r0 + (size_t)a.stats_rows * a.Ngemm;
                *(f32x4 *)r0 = f32x4{ssum[nc][0], ssum[nc][1], ssum[nc][2], ssum[nc][3]};
                *(f32x4 *)(r0 + 4) = f32x4{ssum[nc][4], ssum[nc][5], ssum[nc][6], ssum[nc][7]};
                *(f32x4 *)r1 = f32x4{ssq[nc][0], ssq[nc][1], ssq[nc][2], ssq[nc][3]};
                *(f32x4 *)(r1 + 4) = f32x4{ssq[nc][4], ssq[nc][5], ssq[nc][6], ssq[nc][7]};
            }
        }
    }
}

int tile_rows(const IgemmArgs &a) { return a.Ktot >= 256 ? 32 : 64; }

size_t pw_smem(const IgemmArgs &a, int tm)
{
    return (size_t)a.Ngemm * (a.Ktot * 2 + 16) +
           4 * (size_t)(32 * (a.accumulate ? PW_SROW_F32 : PW_SROW) + (2 * a.ntaps + 2) * tm * 4);
}

template <int KS, int FM, int TAPS, bool ACC> int launch_pw_acc(const PwArgs &pa, hipStream_t stream)
{
    // at least half of a CU's LDS, so that the 256 blocks land on 256 different CUs
    size_t smem = pw_smem(pa.g, 32 * FM);
    if (smem < 84 * 1024) smem = 84 * 1024;
    static bool configured = false;   // the attribute is a property of the function, set once per process
    if (!configured) {
        const hipError_t e = hipFuncSetAttribute((const void *)conv_pw_kernel<KS, FM, TAPS, ACC>,
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) {
            set_last_hip_error(e);
            return NSK_ERR_HIP;
        }
        configured = true;
    }
    hipLaunchKernelGGL((conv_pw_kernel<KS, FM, TAPS, ACC>), dim3(kPwGrid), dim3(256), smem, stream, pa);
    return check_launch();
}

template <int KS, int FM, int TAPS> int launch_pw(const PwArgs &pa, hipStream_t stream)
{
    return pa.g.accumulate ? launch_pw_acc<KS, FM, TAPS, true>(pa, stream) : launch_pw_acc<KS, FM, TAPS, false>(pa, stream);
}

}  // namespace

bool conv_pw_applicable(int dtype, const IgemmArgs &a)
{
    if (getenv("NSK_NO_PW")) return false;
    if (dtype != NSK_BF16 || (a.accumulate && (a.stats || a.zero_cell))) return false;
    if (a.Ktot != a.ntaps * a.Cs || a.Ngemm % 64 != 0 || a.Ngemm > 64 * PW_MAX_NCH) return false;
    if (a.ntaps == 9) {
        // a whole 3x3 filter on 64 -> 64 channels (the stride-2 layer: stride 1 has a kernel that reuses the halo)
        if (a.Cs != 64 || a.Ngemm != 64 || (a.mult_h == 1 && a.mult_w == 1)) return false;
    } else {
        if (!(a.ntaps == 1 || a.ntaps == 2 || a.ntaps == 4)) return false;
        if (!(a.Cs == 64 || a.Cs == 128 || a.Cs == 256) || a.Ktot > 256 || (long)a.Ngemm * a.Ktot > 32768) return false;
    }
    if (a.Co % 8 != 0 || (uintptr_t)a.out % 16 != 0 || (uintptr_t)a.src % 16 != 0 || (uintptr_t)a.wpk % 16 != 0) return false;
    // 32-bit byte offsets below the out-of-range marker
    if ((long)a.Nimg * a.Ho * a.Wo * a.Co * 2 >= (long)PW_OOB || (long)a.src_bytes >= (long)PW_OOB) return false;
    // exact magic-number division of a row index by Mi*Mj and of the remainder by Mj
    if ((long)a.M * a.Mi * a.Mj >= (1L << 40) || (long)a.Mi * a.Mj * a.Mj >= (1L << 40)) return false;
    // enough tiles to give every wavefront of the grid a few (below that the generic kernel's many small blocks win)
    const char *e = getenv("NSK_PW_MIN_ROWS");   // test hook
    const long min_rows = e ? atol(e) : 4L * kPwGrid * 4 * 64;
    return a.M >= min_rows;
}

int conv_pw_stats_rows(const IgemmArgs &) { return kPwGrid * 4; }

int launch_conv_pw(const IgemmArgs &a, hipStream_t stream)
{
    PwArgs pa;
    pa.g = a;
    const int tm = tile_rows(a);
    pa.tiles = ceil_div(a.M, tm);
    pa.zero_cell = a.zero_cell;
    pa.out_bytes = (unsigned)((long)a.Nimg * a.Ho * a.Wo * a.Co * 2);
    const unsigned long long one = 1ull << 40;
    const unsigned long long per_img = (unsigned long long)a.Mi * a.Mj;
    pa.magic_img = (one + per_img - 1) / per_img;
    pa.magic_row = (one + a.Mj - 1) / a.Mj;
    switch (a.Ktot / 16 * 8 + a.ntaps) {   // (k-steps, taps)
    case 4 * 8 + 1: return launch_pw<4, 2, 1>(pa, stream);
    case 8 * 8 + 1: return launch_pw<8, 2, 1>(pa, stream);
    case 8 * 8 + 2: return launch_pw<8, 2, 2>(pa, stream);
    case 16 * 8 + 1: return launch_pw<16, 1, 1>(pa, stream);
    case 16 * 8 + 2: return launch_pw<16, 1, 2>(pa, stream);
    case 16 * 8 + 4: return launch_pw<16, 1, 4>(pa, stream);
    case 36 * 8 + 9: return launch_pw<36, 1, 9>(pa, stream);
    default: return NSK_ERR_UNSUPPORTED;
    }
}

}  // namespace nsk

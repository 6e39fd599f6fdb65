// Kernel template of the short-reduction convolution (see conv_pw.hip for the description); included by the
// translation units that instantiate it (64-channel output chunks in conv_pw.hip, 16- and 32-channel outputs in
// conv_pw_narrow16.hip and conv_pw_narrow32.hip), so that they compile side by side.
#pragma once
#include <stdlib.h>

#include "nsk_internal.h"

namespace nsk {

struct PwArgs {
    IgemmArgs g;
    int tiles;
    int zero_cell;   // also write zeros to the other pixels of each row's 2x2 output cell (see IgemmArgs::zero_cell)
    // Wide outputs whose filter does not fit in LDS are split into col_groups column groups of `cols` channels: a block
    // keeps one group's filter and walks over the tiles of its share of the rows (col_groups divides 32; 1 = no split).
    int cols, col_groups;
    unsigned out_bytes;
    unsigned long long magic_img, magic_row;   // ceil(2^40 / (Mi*Mj)), ceil(2^40 / Mj)
};
// outputs of 16 and of 32 channels (instantiated in conv_pw_narrow16.hip / conv_pw_narrow32.hip); NSK_ERR_UNSUPPORTED for
// a shape without an instance
int launch_conv_pw_narrow16(const PwArgs &pa, hipStream_t stream);
int launch_conv_pw_narrow32(const PwArgs &pa, hipStream_t stream);
// (k-steps, taps) pairs the narrow translation units instantiate
inline bool conv_pw_narrow_instance(int ks, int taps)
{
    const int kpt = taps > 0 && ks % taps == 0 ? ks / taps : 0;     // 16-channel steps per tap
    if (!(taps == 1 || taps == 2 || taps == 4 || taps == 9)) return false;
    return kpt == 1 || kpt == 2 || (kpt == 4 && taps != 9);
}

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kPwGrid = 256;            // blocks; fixed so that the number of statistics rows is a shape property
constexpr unsigned PW_OOB = 0xF0000000u;  // beyond every buffer: loads return zero, stores are dropped
constexpr int PW_MAX_NCH = 4;           // column chunks of 64 (Ngemm <= 256)

template <int KS, int FM, int TAPS, bool ACC, int NW>
__global__ __launch_bounds__(256, 1) void conv_pw_kernel(const PwArgs pa)
{
    const IgemmArgs &a = pa.g;
    constexpr int TM = 32 * FM;                      // pixels per wavefront tile
    constexpr int RPL = (TM + 63) / 64;              // tile rows decoded per lane
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int KPT = KS / TAPS;                   // k-steps (16 channels) per tap
    // Output channels are handled in chunks of NW (64, or the whole of a 32- or 16-channel output).
    constexpr int FN = NW == 64 ? 2 : 1;             // 32-channel MFMA tiles per chunk
    constexpr int SROW = NW * 2 + 16;                // staged bytes per pixel: NW channels and a 16-byte pad
    constexpr int SROW_F32 = NW * 4 + 16;            // the same for fp32 sums (accumulating launches)
    constexpr int CPP = NW / 8;                      // 16-byte pieces of a pixel's chunk
    constexpr int JJ = 32 * CPP / 64 > 0 ? 32 * CPP / 64 : 1;   // pieces per lane and 32-pixel fragment
    constexpr int STRIP = ACC ? 32 * SROW_F32 : 32 * SROW;      // bytes of the transposing strip
    const int Cs = 16 * KPT;
    const int WROW = KS * 32 + 16;                   // filter row pitch: 16 bytes of padding spread the rows over the banks
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int frow = lane & 31, fk = lane >> 5;
    unsigned char *w_lds = smem;
    const int w_rows = pa.cols < 32 ? 32 : pa.cols;   // filter rows in LDS (a 16-channel output still multiplies 32: the rest are zero)
    unsigned char *my_st = smem + (size_t)w_rows * WROW + wave * (STRIP + (2 * TAPS + 2) * TM * 4);
    unsigned *soff_lds = (unsigned *)(my_st + STRIP);   // [2][TAPS][TM] byte offsets of the tile's source pixels
    unsigned *ooff_lds = soff_lds + 2 * TAPS * TM;             // [2][TM] byte offsets of its output pixels (+ flags)

    const __amdgpu_buffer_rsrc_t src_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.src, 0, a.src_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t wpk_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.wpk, 0, a.wpk_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t out_rsrc = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, pa.out_bytes, 0x00020000);

    // filter -> LDS
    // block id -> (column group, row share).  Consecutive ids go to different XCDs, so the column groups of one row
    // share get ids that differ by a multiple of 8: they read the same pixels through one XCD's L2.
    const int cg = ((int)blockIdx.x >> 3) % pa.col_groups;
    const int rb = ((int)blockIdx.x & 7) + 8 * (((int)blockIdx.x >> 3) / pa.col_groups);
    const int n_rb = (int)gridDim.x / pa.col_groups;      // row shares
    const int col0 = cg * pa.cols;                        // first output channel of this block
    for (int idx = tid; idx < w_rows * (2 * KS); idx += 256) {
        const int n = idx / (2 * KS), ch = idx % (2 * KS);
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(wpk_rsrc, n < pa.cols ? (unsigned)(((col0 + n) * KS * 16 + ch * 8) * 2) : PW_OOB, 0, 0);
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
    u32x4 O[2][FM][JJ];
    auto issue_old = [&](u32x4 (&Ob)[FM][JJ], int par, int nc) {
#pragma unroll
        for (int mi = 0; mi < FM; ++mi)
#pragma unroll
            for (int jj = 0; jj < JJ; ++jj) {
                const int idx = lane + 64 * jj, pos = idx / CPP, ck = idx % CPP;
                const unsigned oo = ooff_lds[par * TM + 32 * mi + pos] & ~15u;
                Ob[mi][jj] = __builtin_amdgcn_raw_buffer_load_b128(out_rsrc, oo + (unsigned)((col0 + nc * NW + ck * 8) * 2), 0, 0);
            }
    };

    float ssum[PW_MAX_NCH][8], ssq[PW_MAX_NCH][8];
#pragma unroll
    for (int nc = 0; nc < PW_MAX_NCH; ++nc)
#pragma unroll
        for (int e = 0; e < 8; ++e) ssum[nc][e] = ssq[nc][e] = 0.f;
    const int nch = pa.cols / NW;
    const bool want_stats = a.stats != nullptr;

    auto compute = [&](const u32x4 (&A)[FM][KS], int par, bool has_next) {
#pragma unroll
        for (int nc = 0; nc < PW_MAX_NCH; ++nc) {
            if (nc >= nch) break;
            if constexpr (ACC) {
                if (nc + 1 < nch) issue_old(O[(nc + 1) & 1], par, nc + 1);
            }
            f32x16 acc[FM][FN];
#pragma unroll
            for (int mi = 0; mi < FM; ++mi)
#pragma unroll
                for (int ni = 0; ni < FN; ++ni)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;
            const unsigned char *wb = w_lds + (nc * NW + frow) * WROW + fk * 16;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                bf16x8 bfr[FN];
#pragma unroll
                for (int ni = 0; ni < FN; ++ni) bfr[ni] = *(const bf16x8 *)(wb + ni * 32 * WROW + ks * 32);
#pragma unroll
                for (int mi = 0; mi < FM; ++mi) {
                    const bf16x8 av = __builtin_bit_cast(bf16x8, A[mi][ks]);
#pragma unroll
                    for (int ni = 0; ni < FN; ++ni)
                        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ni], av, acc[mi][ni], 0, 0, 0);
                }
            }
            // acc[mi][ni][4g+j] = channel NW*nc + 32ni + 8g + 4fk + j of pixel 32mi + frow: round, transpose 32 pixels x NW
            // channels through the strip, store the chunk of a pixel (128, 64 or 32 bytes) with CPP lanes.
#pragma unroll
            for (int mi = 0; mi < FM; ++mi) {
#pragma unroll
                for (int ni = 0; ni < FN; ++ni)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        if (ni * 32 + g * 8 >= NW) continue;      // a 16-channel output uses half of the MFMA tile
                        if constexpr (ACC) {
                            *(f32x4 *)(my_st + frow * SROW_F32 + (ni * 32 + g * 8 + fk * 4) * 4) =
                                f32x4{acc[mi][ni][g * 4], acc[mi][ni][g * 4 + 1], acc[mi][ni][g * 4 + 2], acc[mi][ni][g * 4 + 3]};
                        } else {
                            bf16x4 pk;
#pragma unroll
                            for (int j = 0; j < 4; ++j) pk[j] = (bf16_t)acc[mi][ni][g * 4 + j];
                            *(bf16x4 *)(my_st + frow * SROW + (ni * 32 + g * 8 + fk * 4) * 2) = pk;
                        }
                    }
#pragma unroll
                for (int jj = 0; jj < JJ; ++jj) {
                    const int idx = lane + 64 * jj, pos = idx / CPP, ck = idx % CPP;
                    u32x4 v;
                    if constexpr (ACC) {
                        // old value + sum of products, rounded to the storage type once
                        const f32x4 lo = *(const f32x4 *)(my_st + pos * SROW_F32 + ck * 32);
                        const f32x4 hi = *(const f32x4 *)(my_st + pos * SROW_F32 + ck * 32 + 16);
                        const bf16x8 old = __builtin_bit_cast(bf16x8, O[nc & 1][mi][jj]);
                        bf16x8 r;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            r[e] = (bf16_t)(lo[e] + (float)old[e]);
                            r[e + 4] = (bf16_t)(hi[e] + (float)old[e + 4]);
                        }
                        v = __builtin_bit_cast(u32x4, r);
                    } else {
                        v = *(const u32x4 *)(my_st + pos * SROW + ck * 16);
                    }
                    const unsigned oraw = ooff_lds[par * TM + 32 * mi + pos];
                    const unsigned oo = oraw & ~15u, cb = (unsigned)((col0 + nc * NW + ck * 8) * 2);
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
    const int stride = n_rb * 4;
    // few tiles: spread them over the CUs first (one wavefront per CU) instead of filling the first blocks
    int t = pa.tiles >= stride ? rb * 4 + wave : wave * n_rb + rb;
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
        // lanes with equal (lane % CPP) hold the same channels: add them up, one row of partial sums per wavefront
        const int row = rb * 4 + wave, ck = lane % CPP;
#pragma unroll
        for (int nc = 0; nc < PW_MAX_NCH; ++nc) {
            if (nc >= nch) break;
#pragma unroll
            for (int e = 0; e < 8; ++e)
#pragma unroll
                for (int o = CPP; o < 64; o <<= 1) {
                    ssum[nc][e] += __shfl_xor(ssum[nc][e], o, 64);
                    ssq[nc][e] += __shfl_xor(ssq[nc][e], o, 64);
                }
            if (lane < CPP) {
                float *r0 = a.stats + (size_t)row * a.Ngemm + col0 + nc * NW + ck * 8;
                float *r1 = r0 + (size_t)a.stats_rows * a.Ngemm;
                *(f32x4 *)r0 = f32x4{ssum[nc][0], ssum[nc][1], ssum[nc][2], ssum[nc][3]};
                *(f32x4 *)(r0 + 4) = f32x4{ssum[nc][4], ssum[nc][5], ssum[nc][6], ssum[nc][7]};
                *(f32x4 *)r1 = f32x4{ssq[nc][0], ssq[nc][1], ssq[nc][2], ssq[nc][3]};
                *(f32x4 *)(r1 + 4) = f32x4{ssq[nc][4], ssq[nc][5], ssq[nc][6], ssq[nc][7]};
            }
        }
    }
}

inline int pw_chunk(const IgemmArgs &a) { return a.Ngemm % 64 == 0 ? 64 : a.Ngemm; }   // NW: 64, 32 or 16

// Output channels per block: all of them if their filter fits in LDS, else the largest multiple of 64 that does and
// splits the columns into 2, 4, ... 32 groups; 0 if there is none.
inline int pw_cols(const IgemmArgs &a)
{
    const long limit = a.ntaps == 9 ? 36864 : 32768;       // filter elements a block keeps in LDS
    if (a.Ngemm <= 64 * PW_MAX_NCH && (long)a.Ngemm * a.Ktot <= limit) return a.Ngemm;
    if (a.Ngemm % 64 != 0) return 0;
    for (int cols = 64 * PW_MAX_NCH; cols >= 64; cols -= 64) {
        if ((long)cols * a.Ktot > limit || a.Ngemm % cols != 0) continue;
        const int groups = a.Ngemm / cols;
        if (groups <= 32 && 32 % groups == 0) return cols;
    }
    return 0;
}

inline size_t pw_smem(const IgemmArgs &a, int tm)
{
    const int nw = pw_chunk(a), cols = pw_cols(a);
    return (size_t)(cols < 32 ? 32 : cols) * (a.Ktot * 2 + 16) +
           4 * (size_t)(32 * (a.accumulate ? nw * 4 + 16 : nw * 2 + 16) + (2 * a.ntaps + 2) * tm * 4);
}

template <int KS, int FM, int TAPS, bool ACC, int NW> int launch_pw_acc(PwArgs pa, hipStream_t stream)
{
    pa.tiles = ceil_div(pa.g.M, 32 * FM);
    pa.cols = pw_cols(pa.g);
    pa.col_groups = pa.g.Ngemm / pa.cols;
    // at least half of a CU's LDS, so that the 256 blocks land on 256 different CUs
    size_t smem = pw_smem(pa.g, 32 * FM);
    if (smem < 84 * 1024) smem = 84 * 1024;
    static bool configured = false;   // the attribute is a property of the function, set once per process
    if (!configured) {
        const hipError_t e = hipFuncSetAttribute((const void *)conv_pw_kernel<KS, FM, TAPS, ACC, NW>,
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) {
            set_last_hip_error(e);
            return NSK_ERR_HIP;
        }
        configured = true;
    }
    hipLaunchKernelGGL((conv_pw_kernel<KS, FM, TAPS, ACC, NW>), dim3(kPwGrid), dim3(256), smem, stream, pa);
    return check_launch();
}

template <int KS, int FM, int TAPS, int NW> int launch_pw(const PwArgs &pa, hipStream_t stream)
{
    return pa.g.accumulate ? launch_pw_acc<KS, FM, TAPS, true, NW>(pa, stream)
                           : launch_pw_acc<KS, FM, TAPS, false, NW>(pa, stream);
}

}  // namespace
}  // namespace nsk

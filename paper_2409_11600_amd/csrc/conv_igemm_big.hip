// Large-tile bf16 implicit GEMM for the wide layers of the bottleneck stages (1x1 and 3x3 convolutions
// with 64..1024 channels; section "Experiments and Discussion" of the paper names the ResNet recipe
// these shapes come from).  Same GEMM view and the same argument block as the generic kernel
// (rows = output pixels, columns = output channels, k = (tap, channel)), built for the case where the
// matrix units, not memory, should be the limit:
//
//   * block tile 256 pixels x 128 channels (or 256 x 64), four wavefronts of 128 x 64 (64 x 64): a
//     wavefront reads 6 operand fragments from LDS per 8 MFMAs, which keeps LDS traffic (fragment reads
//     plus the staging writes) near 60% of what the CU's LDS delivers at the full MFMA rate;
//   * the reduction index advances 64 channels per k-tile and a tap never straddles a k-tile (C % 64 == 0),
//     so tap and channel offset of a k-tile are wavefront-uniform: a gather address is one add plus the
//     select on the row's tap-validity bit; padding is read as zeros through out-of-range buffer offsets;
//   * eight wavefronts with split roles: four only multiply (fragments fetched one step of 8 MFMAs ahead, one by
//     one behind the MFMAs), four only move data (two k-tiles in flight in registers, a third being written to
//     the other LDS buffer); one LDS-only barrier per k-tile, placed before the fourth step so that this step
//     already reads the next buffer;
//   * block ids are swizzled so that the column blocks of one row block run on the same XCD (they share
//     the activation rows through that XCD's L2).
#include <stdlib.h>

#include "nsk_internal.h"

namespace nsk {
namespace {

constexpr int GB_BM = 256;
constexpr int GB_BK = 64;            // bf16 elements per k-tile row (128 bytes)
constexpr int GB_ROW = 144;          // LDS bytes per row: 128 + 16 pad (conflict-free 16-byte reads of consecutive rows)
constexpr unsigned GB_OOB = 0xF0000000u;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int kBigMultiMax = 4;

// One block's work: tile `b` of the launch described by `a` (b runs over tiles_m * tiles_n).
template <int BN>
__device__ __forceinline__ void igemm_big_block(const IgemmArgs &a, const int b, const int tiles_m, const int tiles_n,
                                                const unsigned out_bytes)
{
    constexpr int FM = BN == 128 ? 4 : 2, FN = 2;                 // 32x32 accumulators per wavefront
    constexpr int WM = FM * 32;
    constexpr int A_LD = GB_BM * 8 / 256, B_LD = BN * 8 / 256;    // 16-byte loads per thread and k-tile
    constexpr int BUF = (GB_BM + BN) * GB_ROW;                    // bytes of one LDS buffer (A rows, then B rows)
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned *out_tab = (unsigned *)(smem + 2 * BUF);             // 256 byte offsets of the output rows

    // Eight wavefronts, two per SIMD: 0..3 multiply (fragment reads, MFMAs, epilogue), 4..7 move data (global loads
    // and LDS writes).  A wavefront issues in order, so a load that waits for room in the CU's memory pipeline would
    // hold back every MFMA behind it; with the roles split only the movers wait there.
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const bool mover = wave >= 4;
    const int tid = threadIdx.x & 255;   // index within the role's 256 threads
    const int cw = wave & 3;
    const int wm = BN == 128 ? cw >> 1 : cw, wn = BN == 128 ? cw & 1 : 0;
    const int frow = lane & 31, fk = lane >> 5;
    const int chunk = tid & 7, lrow = tid >> 3;                   // loader role: 16-byte chunk, row within a pass of 32

    // block id -> (row block, column block): consecutive ids go to different XCDs, so the column blocks of a
    // row block are given ids that differ by a multiple of 8
    int mt, nt;
    {
        const int grp = b / (8 * tiles_n), r = b - grp * 8 * tiles_n;
        const int full = tiles_m / 8;   // groups of 8 row blocks; the tail group is laid out plainly
        if (grp < full) {
            mt = grp * 8 + (r & 7);
            nt = r >> 3;
        } else {
            const int rr = b - full * 8 * tiles_n;
            mt = full * 8 + rr / tiles_n;
            nt = rr % tiles_n;
        }
    }
    const int m0 = mt * GB_BM, n0 = nt * BN;

    const __amdgpu_buffer_rsrc_t src_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.src, 0, a.src_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t wpk_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.wpk, 0, a.wpk_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t out_rsrc = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, out_bytes, 0x00020000);

    // lane t keeps the byte shift of tap t; a k-tile fetches its tap's shift with one cross-lane read
    const int my_tap_shift = lane < a.ntaps ? ((int)a.off_h[lane] * a.Ws + (int)a.off_w[lane]) * a.Cs * 2 : 0;

    // the rows this thread gathers (the same in every k-tile): byte offset of the row's base pixel and the
    // bit mask of the taps that fall inside the image
    unsigned a_base[A_LD];
    unsigned long long a_mask[A_LD];
    const int per_img = a.Mi * a.Mj;
#pragma unroll
    for (int u = 0; u < A_LD; ++u) {
        const int m = m0 + lrow + 32 * u;
        const bool ok = m < a.M;
        const int mm = ok ? m : 0;
        const int img = mm / per_img, rem = mm - img * per_img;
        const int i = rem / a.Mj, j = rem - i * a.Mj;
        const int bh = i * a.mult_h + a.add_h, bw = j * a.mult_w + a.add_w;
        a_base[u] = (unsigned)((img * a.Hs + bh) * a.Ws + bw) * (unsigned)(a.Cs * 2) + (unsigned)(chunk * 16);   // wraps for bh, bw < 0; the tap shift wraps it back
        unsigned long long mask = 0;
        if (ok)
            for (int t = 0; t < a.ntaps; ++t) {
                const int h = bh + a.off_h[t], w = bw + a.off_w[t];
                if ((unsigned)h < (unsigned)a.Hs && (unsigned)w < (unsigned)a.Ws) mask |= 1ull << t;
            }
        a_mask[u] = mask;
    }
    if (!mover) {   // output row offsets (one row per multiplying thread)
        const int m = m0 + tid;
        unsigned off = GB_OOB;
        if (m < a.M) {
            const int img = m / per_img, rem = m - img * per_img;
            const int i = rem / a.Mj, j = rem - i * a.Mj;
            off = (unsigned)((img * a.Ho + (i * a.osh + a.oa)) * a.Wo + (j * a.osw + a.ob)) * (unsigned)(a.Co * 2);
        }
        out_tab[tid] = off;
    }
    unsigned b_base[B_LD];
#pragma unroll
    for (int u = 0; u < B_LD; ++u) {
        const int n = n0 + lrow + 32 * u;
        b_base[u] = n < a.Ngemm ? (unsigned)n * (unsigned)(a.Ktot * 2) + (unsigned)(chunk * 16) : GB_OOB;
    }

    const int nk = a.Ktot / GB_BK;
    const int cpt = a.Cs / GB_BK;       // k-tiles per tap
    // two register sets for the k-tiles in flight
    u32x4 ra[2][A_LD], rb[2][B_LD];
    int ld_tap = 0, ld_cc = 0, ld_kt = 0;   // (tap, chunk within tap) of the next k-tile to load
    auto issue_loads = [&](u32x4 (&A)[A_LD], u32x4 (&B)[B_LD]) {
        const bool live = ld_kt < nk;
        const int tap = live ? ld_tap : 0;
        const int shift = __builtin_amdgcn_readlane(my_tap_shift, tap) + ld_cc * (GB_BK * 2);
#pragma unroll
        for (int u = 0; u < A_LD; ++u) {
            const bool ok = live && ((a_mask[u] >> tap) & 1ull);
            A[u] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, ok ? a_base[u] + (unsigned)shift : GB_OOB, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < B_LD; ++u)
            B[u] = __builtin_amdgcn_raw_buffer_load_b128(wpk_rsrc, live ? b_base[u] + (unsigned)(ld_kt * GB_BK * 2) : GB_OOB, 0, 0);
        ++ld_kt;
        if (++ld_cc == cpt) {
            ld_cc = 0;
            ++ld_tap;
        }
    };
    auto store_item = [&](int buf, const u32x4 (&A)[A_LD], const u32x4 (&B)[B_LD], int i) {
        unsigned char *base = smem + buf * BUF;
        if (i < A_LD)
            *(u32x4 *)(base + (lrow + 32 * i) * GB_ROW + chunk * 16) = A[i];
        else
            *(u32x4 *)(base + (GB_BM + lrow + 32 * (i - A_LD)) * GB_ROW + chunk * 16) = B[i - A_LD];
    };
    constexpr int NL = A_LD + B_LD;
    if (mover) {
        // k-tile 0 -> LDS buffer 0, k-tiles 1 and 2 in flight; then per k-tile kt: write k-tile kt+1 into the other
        // buffer, refilling each register with k-tile kt+3 as soon as it has been written out
        issue_loads(ra[0], rb[0]);
        issue_loads(ra[1], rb[1]);
#pragma unroll
        for (int i = 0; i < NL; ++i) store_item(0, ra[0], rb[0], i);
        issue_loads(ra[0], rb[0]);
        __syncthreads();   // out_tab (written by the multiplying wavefronts) and buffer 0
        auto move = [&](int kt, u32x4 (&A)[A_LD], u32x4 (&B)[B_LD]) {
            const bool live = ld_kt < nk;
            const int tap = live ? ld_tap : 0;
            const int shift = __builtin_amdgcn_readlane(my_tap_shift, tap) + ld_cc * (GB_BK * 2);
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                store_item((kt & 1) ^ 1, A, B, i);
                if (i < A_LD) {
                    const bool ok = live && ((a_mask[i] >> tap) & 1ull);
                    A[i] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, ok ? a_base[i] + (unsigned)shift : GB_OOB, 0, 0);
                } else {
                    const int u = i - A_LD;
                    B[u] = __builtin_amdgcn_raw_buffer_load_b128(wpk_rsrc, live ? b_base[u] + (unsigned)(ld_kt * GB_BK * 2) : GB_OOB, 0, 0);
                }
            }
            ++ld_kt;
            if (++ld_cc == cpt) {
                ld_cc = 0;
                ++ld_tap;
            }
            lds_barrier();
        };
        for (int kt = 0; kt < nk; kt += 2) {
            move(kt, ra[1], rb[1]);
            if (kt + 1 < nk) move(kt + 1, ra[0], rb[0]);
        }
        __syncthreads();   // matches the barrier before the epilogue
        return;
    }

    // accumulators: acc[mi][ni][4g+j] is channel 32ni + 8g + 4fk + j of pixel 32mi + frow of the wavefront's
    // sub-tile (filter rows are the MFMA "A" operand)
    f32x16 acc[FM][FN];
    const int wcol0 = n0 + wn * 64;
    __syncthreads();   // out_tab
    if (a.accumulate) {
        // start from the old values: the sum is rounded to bf16 exactly once
#pragma unroll
        for (int mi = 0; mi < FM; ++mi) {
            const unsigned off = out_tab[wm * WM + mi * 32 + frow];
#pragma unroll
            for (int ni = 0; ni < FN; ++ni)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int col = wcol0 + ni * 32 + g * 8 + fk * 4;
                    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
                    const u32x2 old =
                        __builtin_amdgcn_raw_buffer_load_b64(out_rsrc, col < a.Ngemm ? off + (unsigned)(col * 2) : GB_OOB, 0, 0);
                    const bf16x4 ob = __builtin_bit_cast(bf16x4, old);
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[mi][ni][g * 4 + j] = (float)ob[j];
                }
        }
    } else {
#pragma unroll
        for (int mi = 0; mi < FM; ++mi)
#pragma unroll
            for (int ni = 0; ni < FN; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;
    }

    const unsigned fa0 = (unsigned)((wm * WM + frow) * GB_ROW + fk * 16);
    const unsigned fb0 = (unsigned)((GB_BM + wn * 64 + frow) * GB_ROW + fk * 16);
    bf16x8 af[2][FM], bfr[2][FN];
    // fragment i of a step: the FM pixel fragments, then the FN filter fragments
    auto fetch_item = [&](int buf, int ks, int set, int i) {
        const unsigned char *base = smem + buf * BUF + ks * 32;
        if (i < FM)
            af[set][i] = *(const bf16x8 *)(base + fa0 + i * 32 * GB_ROW);
        else
            bfr[set][i - FM] = *(const bf16x8 *)(base + fb0 + (i - FM) * 32 * GB_ROW);
    };
#pragma unroll
    for (int i = 0; i < FM + FN; ++i) fetch_item(0, 0, 0, i);

    // One k-tile = 4 steps of NS = FM*FN MFMAs; the fragments of step s+1 are fetched one by one behind the MFMAs of
    // step s.  The barrier (the movers have completed the other buffer) sits before step 3, whose fetches already
    // read that buffer.
    constexpr int NS = FM * FN, NF = FM + FN;
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
#pragma unroll
        for (int step = 0; step < 4; ++step) {
            const int set = step & 1;
            if (step == 3) lds_barrier();
#pragma unroll
            for (int j = 0; j < NS; ++j) {
                acc[j / FN][j % FN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[set][j % FN], af[set][j / FN], acc[j / FN][j % FN], 0, 0, 0);
#pragma unroll
                for (int i = j; i < NF; i += NS) fetch_item(step == 3 ? buf ^ 1 : buf, (step + 1) & 3, set ^ 1, i);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    __syncthreads();   // every wavefront is done with the operand buffers: they become the epilogue staging area

    // Epilogue: round to bf16, transpose one 32x32 accumulator tile at a time through this wavefront's strip
    // and store 16 contiguous bytes per lane.
    constexpr int SROW = 80;   // 32 channels bf16 + 16 pad
    unsigned char *my_st = smem + cw * (32 * SROW);
    // statistics epilogue (forward with a batch-norm behind it): a lane reads back the same 8 channels of every staged
    // row, adds them up over the rows it stores, and the wavefront leaves one row of partial sums
    float ssum[FN][8], ssq[FN][8];
#pragma unroll
    for (int ni = 0; ni < FN; ++ni)
#pragma unroll
        for (int e = 0; e < 8; ++e) ssum[ni][e] = ssq[ni][e] = 0.f;
#pragma unroll
    for (int mi = 0; mi < FM; ++mi)
#pragma unroll
        for (int ni = 0; ni < FN; ++ni) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                bf16x4 pk;
#pragma unroll
                for (int j = 0; j < 4; ++j) pk[j] = (bf16_t)acc[mi][ni][g * 4 + j];
                *(bf16x4 *)(my_st + frow * SROW + (g * 8 + fk * 4) * 2) = pk;
            }
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
                const int idx = lane + 64 * jj, pos = idx >> 2, ck = idx & 3;
                const u32x4 v = *(const u32x4 *)(my_st + pos * SROW + ck * 16);
                const unsigned off = out_tab[wm * WM + mi * 32 + pos];
                const int col = wcol0 + ni * 32 + ck * 8;
                const bool live = col < a.Ngemm && off != GB_OOB;
                __builtin_amdgcn_raw_buffer_store_b128(v, out_rsrc, live ? off + (unsigned)(col * 2) : GB_OOB, 0, 0);
                if (a.stats && live) {
                    const bf16x8 vb = __builtin_bit_cast(bf16x8, v);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float f = (float)vb[e];
                        ssum[ni][e] += f;
                        ssq[ni][e] += f * f;
                    }
                }
            }
        }
    if (a.stats) {
        const int row = mt * (GB_BM / WM) + wm, ck = lane & 3;
#pragma unroll
        for (int ni = 0; ni < FN; ++ni) {
#pragma unroll
            for (int e = 0; e < 8; ++e)
#pragma unroll
                for (int o = 4; o < 64; o <<= 1) {
                    ssum[ni][e] += __shfl_xor(ssum[ni][e], o, 64);
                    ssq[ni][e] += __shfl_xor(ssq[ni][e], o, 64);
                }
            const int col = wcol0 + ni * 32 + ck * 8;
            if (lane < 4 && col < a.Ngemm) {
                float *r0 = a.stats + (size_t)row * a.Ngemm + col;
                float *r1 = r0 + (size_t)a.stats_rows * a.Ngemm;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    r0[e] = ssum[ni][e];
                    r1[e] = ssq[ni][e];
                }
            }
        }
    }
}

template <int BN>
__global__ __launch_bounds__(512) void igemm_big_kernel(const IgemmArgs a, const int tiles_m, const int tiles_n,
                                                        const unsigned out_bytes)
{
    igemm_big_block<BN>(a, blockIdx.x, tiles_m, tiles_n, out_bytes);
}

// Several launches in one: the residue classes of a strided backward-data pass (same source, same output tensor, same
// column count; each class with its own taps, filter and row count).  Each class alone leaves part of the chip idle
// and pays its own start-up; together their tiles fill it.  Block ids are assigned class by class, longest reduction
// first.
struct BigMulti {
    IgemmArgs a[kBigMultiMax];
    int first[kBigMultiMax + 1];   // first block id of each class
    int tiles_m[kBigMultiMax];
    int count;
};

template <int BN>
__global__ __launch_bounds__(512) void igemm_big_multi_kernel(const BigMulti m, const int tiles_n, const unsigned out_bytes)
{
    int cls = 0;
    while (cls + 1 < m.count && (int)blockIdx.x >= m.first[cls + 1]) ++cls;
    igemm_big_block<BN>(m.a[cls], (int)blockIdx.x - m.first[cls], m.tiles_m[cls], tiles_n, out_bytes);
}

template <int BN> int smem_bytes() { return 2 * (GB_BM + BN) * GB_ROW + 256 * 4; }

}  // namespace

bool igemm_big_applicable(int dtype, const IgemmArgs &a)
{
    if (dtype != NSK_BF16 || hooks().no_big) return false;
    if (a.Cs % GB_BK != 0 || a.Ngemm % 64 != 0 || a.Co % 8 != 0 || a.ntaps > 64 || a.ntaps < 1) return false;
    if (((uintptr_t)a.src | (uintptr_t)a.wpk | (uintptr_t)a.out) & 15) return false;
    const long long out_bytes = (long long)a.Nimg * a.Ho * a.Wo * a.Co * 2;
    if ((unsigned long long)a.src_bytes >= GB_OOB || (unsigned long long)a.wpk_bytes >= GB_OOB || out_bytes >= (long long)GB_OOB)
        return false;
    // Measured against the generic kernel on the bottleneck-stage layers: this one wins when the reduction is long
    // (at least 8 k-tiles) and there are at least 128 output channels; short reductions and 64-channel outputs are
    // bound by memory and do better with the generic kernel's several small blocks per CU.  The 256-row tiles must
    // also still fill the chip.  NSK_BIG_MIN_TILES overrides all three tests (tests use it to run small shapes
    // through this kernel).
    const long long tiles = (long long)ceil_div(a.M, GB_BM) * ceil_div(a.Ngemm, a.Ngemm >= 128 ? 128 : 64);
    if (hooks().big_min_tiles >= 0) return tiles >= hooks().big_min_tiles;
    return tiles >= 160 && a.Ngemm >= 128 && a.Ktot >= 8 * GB_BK;
}

// Rows of partial sums the forward launch writes: one per multiplying wavefront row of every row block.
int igemm_big_stats_rows(const IgemmArgs &a)
{
    const int wm = a.Ngemm >= 128 ? 128 : 64;
    return ceil_div(a.M, GB_BM) * (GB_BM / wm);
}

int launch_igemm_big(const IgemmArgs &a, hipStream_t stream)
{
    const int bn = a.Ngemm >= 128 ? 128 : 64;
    const int tiles_m = ceil_div(a.M, GB_BM), tiles_n = ceil_div(a.Ngemm, bn);
    const unsigned out_bytes = (unsigned)((long long)a.Nimg * a.Ho * a.Wo * a.Co * 2);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)igemm_big_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           smem_bytes<128>());
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)igemm_big_kernel<64>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes<64>());
        if (e != hipSuccess) {
            set_last_hip_error(e);
            return NSK_ERR_HIP;
        }
        attr_set = true;
    }
    const dim3 grid((unsigned)(tiles_m * tiles_n));
    if (bn == 128)
        hipLaunchKernelGGL(igemm_big_kernel<128>, grid, dim3(512), smem_bytes<128>(), stream, a, tiles_m, tiles_n, out_bytes);
    else
        hipLaunchKernelGGL(igemm_big_kernel<64>, grid, dim3(512), smem_bytes<64>(), stream, a, tiles_m, tiles_n, out_bytes);
    return check_launch();
}


// The shape tests of igemm_big_applicable without its size thresholds.
static bool big_shape_ok(const IgemmArgs &a)
{
    if (a.Cs % GB_BK != 0 || a.Ngemm % 64 != 0 || a.Co % 8 != 0 || a.ntaps > 64 || a.ntaps < 1) return false;
    if (((uintptr_t)a.src | (uintptr_t)a.wpk | (uintptr_t)a.out) & 15) return false;
    const long long out_bytes = (long long)a.Nimg * a.Ho * a.Wo * a.Co * 2;
    return (unsigned long long)a.src_bytes < GB_OOB && (unsigned long long)a.wpk_bytes < GB_OOB && out_bytes < (long long)GB_OOB;
}

bool igemm_big_multi_applicable(int dtype, const IgemmArgs *a, int count)
{
    if (dtype != NSK_BF16 || hooks().no_big || hooks().no_big_multi) return false;
    if (count < 2 || count > kBigMultiMax) return false;
    long long tiles = 0;
    int longest = 0;
    for (int i = 0; i < count; ++i) {
        if (!big_shape_ok(a[i]) || a[i].stats || a[i].zero_cell) return false;
        if (a[i].Ngemm != a[0].Ngemm || a[i].out != a[0].out || a[i].Co != a[0].Co || a[i].Nimg != a[0].Nimg ||
            a[i].Ho != a[0].Ho || a[i].Wo != a[0].Wo)
            return false;
        tiles += (long long)ceil_div(a[i].M, GB_BM) * ceil_div(a[i].Ngemm, a[i].Ngemm >= 128 ? 128 : 64);
        if (a[i].Ktot > longest) longest = a[i].Ktot;
    }
    if (hooks().big_min_tiles >= 0) return tiles >= hooks().big_min_tiles;   // test hook, as in igemm_big_applicable
    return tiles >= 160 && a[0].Ngemm >= 128 && longest >= 8 * GB_BK;
}

int launch_igemm_big_multi(const IgemmArgs *a, int count, hipStream_t stream)
{
    const int bn = a[0].Ngemm >= 128 ? 128 : 64;
    const int tiles_n = ceil_div(a[0].Ngemm, bn);
    // longest reduction first
    int order[kBigMultiMax];
    for (int i = 0; i < count; ++i) order[i] = i;
    for (int i = 1; i < count; ++i)
        for (int j = i; j > 0 && a[order[j]].Ktot > a[order[j - 1]].Ktot; --j) {
            const int t = order[j];
            order[j] = order[j - 1];
            order[j - 1] = t;
        }
    BigMulti m{};
    m.count = count;
    int blocks = 0;
    for (int i = 0; i < count; ++i) {
        m.a[i] = a[order[i]];
        m.tiles_m[i] = ceil_div(m.a[i].M, GB_BM);
        m.first[i] = blocks;
        blocks += m.tiles_m[i] * tiles_n;
    }
    m.first[count] = blocks;
    const unsigned out_bytes = (unsigned)((long long)a[0].Nimg * a[0].Ho * a[0].Wo * a[0].Co * 2);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)igemm_big_multi_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes<128>());
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)igemm_big_multi_kernel<64>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes<64>());
        if (e != hipSuccess) {
            set_last_hip_error(e);
            return NSK_ERR_HIP;
        }
        attr_set = true;
    }
    if (bn == 128)
        hipLaunchKernelGGL(igemm_big_multi_kernel<128>, dim3(blocks), dim3(512), smem_bytes<128>(), stream, m, tiles_n, out_bytes);
    else
        hipLaunchKernelGGL(igemm_big_multi_kernel<64>, dim3(blocks), dim3(512), smem_bytes<64>(), stream, m, tiles_n, out_bytes);
    return check_launch();
}

}  // namespace nsk

// Backward-weight convolution for the wide bf16 layers (channel counts that are multiples of 64; the 1x1
// and 3x3 layers of the bottleneck stages of the ResNet recipe the paper trains, section "Experiments and
// Discussion"; the gradient is the one the paper accumulates into its gradient cache, section "Caching and
// Pooling").
//
//   dw[k][tap][c] = sum over output pixels l of dy[l][k] * x[pixel(l) shifted by tap][c]
//
// GEMM view: rows = output channels k, columns n = (tap, input channel), reduction over the N*P*Q output
// pixels, split across blocks into fp32 partials that the fixed-order reduce kernel adds (bitwise
// reproducible, no floating-point atomics).
//
// These layers are bound by memory, not by the matrix units, so the kernel is built around traffic:
//   * a block owns a 256 x 128 (or 64 x 128) tile of dw: dy is read once per column tile and x once per row
//     tile, and the number of splits is chosen so that one launch is about one block per CU - the partial
//     sums written and re-read are then blocks x tile bytes, a fraction of the operand bytes;
//   * both operands are copied to LDS exactly as they lie in memory ([pixel][channel], 16-byte pieces) and
//     come out through the transposing LDS read, which delivers 8 consecutive pixels of one channel per lane
//     (the MFMA operand layout) without any 2-byte shuffling;
//   * eight wavefronts with split roles: four only multiply (fragment reads + MFMAs), four only move data
//     (two k-tiles of 64 pixels in flight in registers, a third being written to the other LDS buffer); one
//     LDS-only barrier per k-tile;
//   * the tiles of one split get block ids that land on the same XCD, so its dy and x rows are shared
//     through that XCD's L2.
#include <stdlib.h>

#include "nsk_internal.h"

namespace nsk {
namespace {

constexpr int WW_BN = 128;            // columns of a tile
constexpr int WW_KT = 64;             // pixels per k-tile
constexpr int WW_XROW = 2 * WW_BN + 64;   // LDS bytes per pixel row of the x tile (pad: conflict-free transposing reads)
constexpr unsigned WW_OOB = 0xF0000000u;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct WWArgs {
    WgradArgs g;
    int tiles_n, tiles_k;
    unsigned long long magic_pq, magic_q;   // ceil(2^40 / (P*Q)), ceil(2^40 / Q)
    unsigned x_bytes, dy_bytes;
};

template <int FM>   // 32-row accumulator tiles per wavefront in k: block rows = 64 * FM
__global__ __launch_bounds__(512) void wgrad_wide_kernel(const WWArgs w)
{
    const WgradArgs &a = w.g;
    constexpr int BM = 64 * FM;
    constexpr int DROW = 2 * BM + 64;               // LDS bytes per pixel row of the dy tile
    constexpr int D_CPR = BM / 8;                   // 16-byte chunks per dy row
    constexpr int D_RPP = 256 / D_CPR;              // dy rows per pass of the 256 threads
    constexpr int D_LD = WW_KT / D_RPP;             // dy loads per thread and k-tile
    constexpr int X_LD = WW_KT * (WW_BN / 8) / 256; // x loads per thread and k-tile (4)
    constexpr int BUF = WW_KT * (DROW + WW_XROW);
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    // Eight wavefronts, two per SIMD: 0..3 multiply (fragment reads and MFMAs only), 4..7 move data (global loads
    // and LDS writes only).  A wavefront issues in order, so a load that waits for room in the CU's memory pipeline
    // would hold back every MFMA behind it; with the roles split, only the movers ever wait there.
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const bool mover = wave >= 4;
    const int tid = threadIdx.x & 255;   // index within the role's 256 threads
    const int wm = (wave & 3) >> 1, wn = wave & 1;
    const int frow = lane & 31, fk = lane >> 5;

    // block id -> (split, tile): within a group of 8 splits the split index is the fastest, so the tiles of a
    // split run on one XCD
    const int T = w.tiles_n * w.tiles_k;
    int split, tile;
    {
        const int b = blockIdx.x, full = a.splits / 8;
        const int grp = b / (8 * T);
        if (grp < full) {
            const int r = b - grp * 8 * T;
            split = grp * 8 + (r & 7);
            tile = r >> 3;
        } else {
            const int rem = a.splits - full * 8, r = b - full * 8 * T;
            split = full * 8 + r % rem;
            tile = r / rem;
        }
    }
    const int n0 = (tile % w.tiles_n) * WW_BN, k0 = (tile / w.tiles_n) * BM;
    const int NT = a.ntaps * a.C;
    const int l_begin = split * a.rows_per_split;
    const int l_end = min(a.L, l_begin + a.rows_per_split);
    const int nk = (l_end - l_begin + WW_KT - 1) / WW_KT;

    const __amdgpu_buffer_rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, w.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t dy_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.dy, 0, w.dy_bytes, 0x00020000);

    // loader roles
    const int d_chunk = tid % D_CPR, d_row = tid / D_CPR;
    const int x_chunk = tid & 15, x_row = tid >> 4;
    const int d_k = k0 + d_chunk * 8;
    // this thread's x column: a fixed (tap, channel)
    const int x_n = n0 + x_chunk * 8;
    const bool x_live = x_n < NT;
    const int x_tap = x_live ? x_n / a.C : 0;
    const int x_c = x_live ? x_n - x_tap * a.C : 0;
    const int x_oh = a.off_h[x_tap] - a.ph, x_ow = a.off_w[x_tap] - a.pw;

    u32x4 rd[2][D_LD], rx[2][X_LD];
    int ld_l = l_begin;   // first pixel of the next k-tile to load
    // Running addresses, advanced by one k-tile (64 pixels) at a time with adds and selects only (no
    // multiplication, division or branch inside the loop).
    //   dy: byte offset of each row of this thread.
    //   x:  per row the pixel's (p*sh, q*sw) and the byte offset of its tap-shifted source element; 64 pixels
    //       further is adv_q columns and adv_p rows on, with a carry from q into p and up to two from p into
    //       the image index (the applicability test guarantees adv_p + 1 <= 2P).
    unsigned d_off[D_LD];
#pragma unroll
    for (int u = 0; u < D_LD; ++u) d_off[u] = (unsigned)(l_begin + d_row + D_RPP * u) * (unsigned)(a.K * 2) + (unsigned)(d_k * 2);
    const bool d_live = d_k < a.K;
    const unsigned d_step = (unsigned)(WW_KT * a.K * 2);
    int x_hh[X_LD], x_wq[X_LD];
    unsigned x_off[X_LD];
    const unsigned C2 = (unsigned)(a.C * 2);
#pragma unroll
    for (int u = 0; u < X_LD; ++u) {
        const unsigned ll = (unsigned)min(l_begin + x_row + 16 * u, a.L - 1);
        const unsigned img = (unsigned)(((unsigned long long)ll * w.magic_pq) >> 40);
        const unsigned rem = ll - img * (unsigned)(a.P * a.Q);
        const unsigned p = (unsigned)(((unsigned long long)rem * w.magic_q) >> 40);
        const unsigned q = rem - p * (unsigned)a.Q;
        x_hh[u] = (int)p * a.sh;
        x_wq[u] = (int)q * a.sw;
        x_off[u] = ((img * (unsigned)a.H + (unsigned)(x_hh[u] + x_oh)) * (unsigned)a.W + (unsigned)(x_wq[u] + x_ow)) * C2 + (unsigned)(x_c * 2);
    }
    const int adv_p = WW_KT / a.Q, adv_q = WW_KT % a.Q;
    const int Qs = a.Q * a.sw, Ps = a.P * a.sh, aqs = adv_q * a.sw, aps = adv_p * a.sh;
    const unsigned s_q = (unsigned)(aqs + aps * a.W) * C2;             // adv_q columns and adv_p rows on
    const unsigned s_qwrap = (unsigned)(a.sh * a.W - Qs) * C2;         // q wrapped: back Q columns, one row on
    const unsigned s_pwrap = (unsigned)(a.H * a.W - Ps * a.W) * C2;    // p wrapped: back P rows, one image on
    auto load_d = [&](u32x4 (&D)[D_LD], int u) {
        const bool ok = d_live && ld_l + d_row + D_RPP * u < l_end;
        D[u] = __builtin_amdgcn_raw_buffer_load_b128(dy_rsrc, ok ? d_off[u] : WW_OOB, 0, 0);
        d_off[u] += d_step;
    };
    auto load_x = [&](u32x4 (&X)[X_LD], int u) {
        const int h = x_hh[u] + x_oh, ww = x_wq[u] + x_ow;
        const bool ok = x_live & (ld_l + x_row + 16 * u < l_end) & ((unsigned)h < (unsigned)a.H) & ((unsigned)ww < (unsigned)a.W);
        X[u] = __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, ok ? x_off[u] : WW_OOB, 0, 0);
        // advance this row to the next k-tile
        int wq = x_wq[u] + aqs, hh = x_hh[u] + aps;
        unsigned off = x_off[u] + s_q;
        const bool c1 = wq >= Qs;
        wq -= c1 ? Qs : 0;
        hh += c1 ? a.sh : 0;
        off += c1 ? s_qwrap : 0u;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const bool c2 = hh >= Ps;
            hh -= c2 ? Ps : 0;
            off += c2 ? s_pwrap : 0u;
        }
        x_wq[u] = wq;
        x_hh[u] = hh;
        x_off[u] = off;
    };
    // work item i of a k-tile's loads (dy first, then x); ld_l moves on once all items of the k-tile are issued
    auto load_item = [&](u32x4 (&D)[D_LD], u32x4 (&X)[X_LD], int i) {
        if (i < D_LD)
            load_d(D, i);
        else
            load_x(X, i - D_LD);
    };
    auto issue_loads = [&](u32x4 (&D)[D_LD], u32x4 (&X)[X_LD]) {
#pragma unroll
        for (int i = 0; i < D_LD + X_LD; ++i) load_item(D, X, i);
        ld_l += WW_KT;
    };
    auto store_item = [&](int buf, const u32x4 (&D)[D_LD], const u32x4 (&X)[X_LD], int i) {
        unsigned char *base = smem + buf * BUF;
        if (i < D_LD)
            *(u32x4 *)(base + (d_row + D_RPP * i) * DROW + d_chunk * 16) = D[i];
        else
            *(u32x4 *)(base + WW_KT * DROW + (x_row + 16 * (i - D_LD)) * WW_XROW + x_chunk * 16) = X[i - D_LD];
    };

    constexpr int NL = D_LD + X_LD;
    if (mover) {
        // k-tile 0 -> LDS buffer 0, k-tiles 1 and 2 in flight; then per k-tile kt: write k-tile kt+1 into the other
        // buffer and refill each register with k-tile kt+3 as soon as it has been written out (measured faster than
        // all writes followed by all loads, and than a third register set with the loads issued first)
        issue_loads(rd[0], rx[0]);
        issue_loads(rd[1], rx[1]);
#pragma unroll
        for (int i = 0; i < NL; ++i) store_item(0, rd[0], rx[0], i);
        issue_loads(rd[0], rx[0]);
        lds_barrier();
        auto move = [&](int kt, u32x4 (&D)[D_LD], u32x4 (&X)[X_LD]) {
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                store_item((kt & 1) ^ 1, D, X, i);
                load_item(D, X, i);
            }
            ld_l += WW_KT;
            lds_barrier();
        };
        for (int kt = 0; kt < nk; kt += 2) {
            move(kt, rd[1], rx[1]);
            if (kt + 1 < nk) move(kt + 1, rd[0], rx[0]);
        }
        return;
    }

    f32x16 acc[FM][2];
#pragma unroll
    for (int mi = 0; mi < FM; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;
    lds_barrier();   // buffer 0 is ready

    // Transposing read: within 16 lanes, lanes 4j..4j+3 address row j (four 8-byte pieces = 16 channels) and lane
    // i receives channel i of rows 0..3.  Lane (channel = lane%32, half = lane/32) of an MFMA operand needs pixels
    // 8*half .. 8*half+7 of its channel: two such reads, four pixel rows apart.
    const int g16 = lane >> 4, i16 = lane & 15;
    const unsigned tr_row = (unsigned)(8 * (g16 >> 1) + (i16 >> 2)), tr_col = (unsigned)((16 * (g16 & 1) + 4 * (i16 & 3)) * 2);
    const unsigned fd0 = tr_row * DROW + tr_col + (unsigned)(wm * 32 * FM * 2);
    const unsigned fx0 = (unsigned)(WW_KT * DROW) + tr_row * WW_XROW + tr_col + (unsigned)(wn * 64 * 2);
    typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
    auto tr8 = [&](const unsigned char *p, int row_bytes) -> bf16x8 {
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)(p));
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)(p + 4 * row_bytes));
        bf16x8 r;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            r[e] = lo[e];
            r[4 + e] = hi[e];
        }
        return r;
    };
    bf16x8 af[2][FM], bfr[2][2];
    // fragment i of a step: the FM dy fragments, then the 2 x fragments
    auto fetch_item = [&](int buf, int ks, int set, int i) {
        const unsigned char *base = smem + buf * BUF;
        if (i < FM)
            af[set][i] = tr8(base + fd0 + ks * 16 * DROW + i * 64, DROW);
        else
            bfr[set][i - FM] = tr8(base + fx0 + ks * 16 * WW_XROW + (i - FM) * 64, WW_XROW);
    };
#pragma unroll
    for (int i = 0; i < FM + 2; ++i) fetch_item(0, 0, 0, i);

    // One k-tile = 4 steps of NS = 2*FM MFMAs; the fragments of step s+1 are fetched one by one behind the MFMAs
    // of step s.  The barrier (the movers have completed the other buffer) sits before step 3, whose fetches
    // already read that buffer.
    constexpr int NS = 2 * FM, NF = FM + 2;
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
#pragma unroll
        for (int step = 0; step < 4; ++step) {
            const int set = step & 1;
            if (step == 3) lds_barrier();
#pragma unroll
            for (int j = 0; j < NS; ++j) {
                acc[j >> 1][j & 1] =
                    __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[set][j >> 1], bfr[set][j & 1], acc[j >> 1][j & 1], 0, 0, 0);
#pragma unroll
                for (int i = j; i < NF; i += NS) fetch_item(step == 3 ? buf ^ 1 : buf, (step + 1) & 3, set ^ 1, i);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    // acc[mi][ni][v]: row k = 32*mi + 8*(v/4) + 4*(lane/32) + v%4, column = 32*ni + lane%32 of the wavefront's sub-tile
    float *__restrict__ part = a.part + (size_t)split * a.K * NT;
#pragma unroll
    for (int mi = 0; mi < FM; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            const int col = n0 + wn * 64 + ni * 32 + frow;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = k0 + wm * 32 * FM + mi * 32 + 8 * (v >> 2) + 4 * fk + (v & 3);
                if (k < a.K && col < NT) part[(size_t)k * NT + col] = acc[mi][ni][v];
            }
        }
}

template <int FM> int smem_bytes() { return 2 * WW_KT * (2 * 64 * FM + 64 + WW_XROW); }

int tile_rows(const WgradArgs &a) { return a.K % 256 == 0 ? 256 : 64; }

}  // namespace

bool wgrad_wide_applicable(int dtype, const WgradArgs &a)
{
    if (dtype != NSK_BF16 || hooks().no_wide) return false;
    // a thread's 8 x-columns must share one tap (C % 8), a dy row is loaded in 16-byte pieces up to the tile height
    // (a tile of 64 rows also serves fewer output channels: the missing rows are neither loaded nor stored)
    if (a.C % 8 != 0 || a.K % 8 != 0 || (a.K % 256 != 0 && a.K > 64)) return false;
    if (((uintptr_t)a.x | (uintptr_t)a.dy) & 15) return false;
    const long long pq = (long long)a.P * a.Q;
    if ((long long)a.L >= (1LL << 30) || (long long)a.L * pq >= (1LL << 40)) return false;   // exactness of the reciprocal division
    const long long xb = (long long)a.Nimg * a.H * a.W * a.C * 2, db = (long long)a.L * a.K * 2;
    if (xb >= (long long)WW_OOB || db >= (long long)WW_OOB) return false;
    if (WW_KT / a.Q + 1 > 2 * a.P) return false;   // the running pixel decode handles at most two image wraps per k-tile
    // a long reduction per block is what pays for the large tile (NSK_WIDE_MIN_ROWS: test hook)
    return a.L >= (hooks().wide_min_rows >= 0 ? hooks().wide_min_rows : 16384);
}

// Number of splits (written to *splits) and rows per split for the wide kernel: about one block per CU.
int wgrad_wide_rows_per_split(const WgradArgs &a, int *splits)
{
    const int NT = a.ntaps * a.C;
    const int T = ceil_div(NT, WW_BN) * ceil_div(a.K, tile_rows(a));
    // The 64-row kernel needs 65 KB of LDS, so two of its blocks can share a CU.  Measured: that pays for long
    // reductions over several taps (image stem 83 -> 71 us, strided 3x3 64->64 82 -> 71 us), whose blocks wait on
    // gathered loads; single-tap layers are bound by HBM and lose (110 -> 117 us), and so do short reductions.
    // (from 200 k rows on: the 16-channel 3x3 layers of the CIFAR-sized network at batch 256 gain too, 0.923 -> 0.915 ms
    // per step; at 65 k rows and below nothing changes)
    int want = (tile_rows(a) == 64 && a.ntaps > 1 && a.L >= 200000 ? 512 : 256) / T;
    if (want < 1) want = 1;
    const int most = ceil_div(a.L, 2 * WW_KT);   // at least two k-tiles per split
    if (want > most) want = most;
    int rows = ceil_div(ceil_div(a.L, want), WW_KT) * WW_KT;
    *splits = ceil_div(a.L, rows);
    return rows;
}

int launch_wgrad_wide(const WgradArgs &a, hipStream_t stream)
{
    WWArgs w{};
    w.g = a;
    const int bm = tile_rows(a);
    w.tiles_n = ceil_div(a.ntaps * a.C, WW_BN);
    w.tiles_k = ceil_div(a.K, bm);
    const unsigned long long pq = (unsigned long long)a.P * a.Q;
    w.magic_pq = ((1ULL << 40) + pq - 1) / pq;
    w.magic_q = ((1ULL << 40) + a.Q - 1) / a.Q;
    w.x_bytes = (unsigned)((long long)a.Nimg * a.H * a.W * a.C * 2);
    w.dy_bytes = (unsigned)((long long)a.L * a.K * 2);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)wgrad_wide_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes<4>());
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)wgrad_wide_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes<1>());
        if (e != hipSuccess) {
            set_last_hip_error(e);
            return NSK_ERR_HIP;
        }
        attr_set = true;
    }
    const dim3 grid((unsigned)(w.tiles_n * w.tiles_k * a.splits));
    if (bm == 256)
        hipLaunchKernelGGL(wgrad_wide_kernel<4>, grid, dim3(512), smem_bytes<4>(), stream, w);
    else
        hipLaunchKernelGGL(wgrad_wide_kernel<1>, grid, dim3(512), smem_bytes<1>(), stream, w);
    return check_launch();
}

}  // namespace nsk

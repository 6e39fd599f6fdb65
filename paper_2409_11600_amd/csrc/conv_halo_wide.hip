// 3x3, stride 1, bf16 convolution with many channels (128, 256 or 512 in, a multiple of 128 out): forward, and
// backward-data through the packed transposed filter.  These are the 3x3 layers of the later bottleneck stages of
// the residual networks the paper trains (section "Experiments and Discussion"); with 2304 or more reduction indices
// they are the layers where the matrix units, not memory, should be the limit.
//
// The large-tile kernel re-stages every activation row nine times (once per tap) and every filter row once per row
// block, all through LDS: 144 KB of LDS traffic and 48 KB of L2 traffic per 1024 MFMA clocks, which holds it below
// 40% MFMA utilisation.  This kernel removes both:
//   * the input tile (whole image rows with their halo, ALL input channels) is staged into LDS once; the nine taps
//     are shifted reads of the same rows (flat padded coordinates: the tile is a run of consecutive positions of the
//     zero-padded image, so a tap is one constant shift and borders need no special case);
//   * the filter never passes through LDS: it is the MFMA "A" operand, each wavefront streams the rows of its 32 output
//     channels straight from L2 into registers, 64 contiguous bytes per lane, tap and 64-channel group, three such
//     pieces in flight.  (The reduction index inside a group is permuted so that those 64 bytes are four operand fragments; the
//     pixel fragments are read from LDS in the same order.)
//   * per 32-clock MFMA the main loop issues one 16-byte LDS read per lane; the tile is staged one 64-channel group at
//     a time by a fifth wavefront, group g+1 while group g is multiplied, so only the first group's loads are exposed
//     (one barrier per group).
// Block = NT*32 positions x 128 output channels, 4 multiplying wavefronts + 1 that moves data; wavefront w < 4 owns channels 32w..32w+31 of all NT position
// tiles (NT accumulators of 32x32).  For 14 x 14 images a tile is exactly one image (14 rows of 16 padded positions).
#include <stdlib.h>

#include "nsk_internal.h"

namespace nsk {
namespace {

constexpr unsigned W_OOB = 0xF0000000u;
constexpr int W_BN = 128;                           // output channels per block
constexpr int W_LDS_MAX = 152 * 1024;               // staged input + output row table
constexpr int W_MAXLD = 36;                         // 16-byte loads the moving wavefront keeps in flight
constexpr int W_THREADS = 320;                      // four multiplying wavefronts and one that moves data
constexpr int W_STAGE_MAX = 576;                    // staged positions of a tile, at most (two rounds of the moving wavefront)
constexpr int W_TAB = 640;                          // entries of the staged-position table (two per thread)
constexpr int W_LD0 = (W_STAGE_MAX * 8 + W_THREADS - 1) / W_THREADS;   // loads per thread for the first group

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

struct WideArgs {
    const void *src, *wpk;
    void *out;
    int N, H, W, C, K, Co;
    int PW;                       // padded width W + 2
    int rows_per_tile, tiles_per_img, tiles;
    int n_stage;                  // staged positions: NT*32 + 2*(PW + 1)
    int row_bytes;                // LDS bytes per staged position: 2*C + 16
    unsigned long long magic_pw;  // ceil(2^40 / PW)
    unsigned src_bytes, wpk_bytes, out_bytes;
    int accumulate;
    int tapbyte[9];               // LDS byte shift of each tap: (PW + 1 + dh*PW + dw) * row_bytes
    float *stats;                 // per-channel partial sums of the stored output (one row per tile), or nullptr
    int stats_rows;
};

template <int NT, bool ACCUM>
__global__ __launch_bounds__(W_THREADS) void conv_halo_wide_kernel(const WideArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char *in_lds = smem;
    unsigned *out_tab = (unsigned *)(smem + a.n_stage * a.row_bytes);   // NT*32 byte offsets of the output rows
    unsigned *in_tab = out_tab + NT * 32;                               // W_TAB byte offsets of the staged positions

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int frow = lane & 31, fk = lane >> 5;

    // block id -> (tile, column block).  Consecutive ids run on different XCDs; with two column blocks an XCD sees
    // only one half of the filter.
    const int tiles_n = a.K / W_BN;
    const int nt = (int)blockIdx.x % tiles_n, tile = (int)blockIdx.x / tiles_n;
    const int img = tile / a.tiles_per_img, r0 = (tile - img * a.tiles_per_img) * a.rows_per_tile;
    const int n0 = nt * W_BN;

    const __amdgpu_buffer_rsrc_t src_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.src, 0, a.src_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t wpk_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.wpk, 0, a.wpk_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t out_rsrc = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, a.out_bytes, 0x00020000);

    const int cpt = a.C >> 6;    // 64-channel groups
    const unsigned tile_step = (unsigned)(32 * a.row_bytes);

    // ---- filter stream (wavefronts 0..3): lane (row r = lane % 32, half h = lane / 32) reads bytes [64h, 64h + 64) of
    // the 128 bytes that one (tap, 64-channel group) occupies in filter row n0 + 32*wave + r.  Groups are the outer
    // loop, taps the inner.  The first three pieces are requested before anything else.
    const unsigned wrow = (unsigned)(n0 + (wave & 3) * 32 + frow) * (unsigned)(9 * a.C * 2) + (unsigned)(fk * 64);
    u32x4 wf[3][4];
    int ld_t = 0, ld_g = 0;      // (tap, group) of the next filter piece to load
    auto load_w = [&](u32x4 (&Wf)[4]) {
        const unsigned off = ld_g < cpt ? wrow + (unsigned)(ld_t * a.C * 2 + ld_g * 128) : W_OOB;
#pragma unroll
        for (int s = 0; s < 4; ++s) Wf[s] = __builtin_amdgcn_raw_buffer_load_b128(wpk_rsrc, off + (unsigned)(s * 16), 0, 0);
        if (++ld_t == 9) {
            ld_t = 0;
            ++ld_g;
        }
    };
    if (wave < 4) {
        load_w(wf[0]);
        load_w(wf[1]);
        load_w(wf[2]);
    }

    // ---- staging.  Staged position s is position r0*PW - 1 + s of the zero-padded image (row-major from the top-left
    // corner of the padding); in_tab[s] is its byte offset in src, or out of range for padding.  The tile is staged
    // one 64-channel group at a time: group 0 by all five wavefronts, group g+1 by the fifth wavefront alone while the
    // other four multiply group g (they meet at one barrier per group).  After the first group no input load is
    // exposed, and the multiplying wavefronts have nothing but their filter stream in their (in-order) load queue.
    // One-time code is kept short on purpose: a block runs once per launch, so all of it is fetched cold.
    for (int s = tid; s < W_TAB; s += W_THREADS) {
        // u counts from one row above the padded image (so that it is never negative): u / PW is the image row + 2,
        // u % PW the image column + 1
        const unsigned u = (unsigned)((r0 + 1) * a.PW - 1 + s);
        const unsigned hp1 = (unsigned)(((unsigned long long)u * a.magic_pw) >> 40);
        const unsigned wp = u - hp1 * (unsigned)a.PW;
        const bool ok = s < a.n_stage && (hp1 - 2u < (unsigned)a.H) && (wp - 1u < (unsigned)a.W);
        in_tab[s] = ok ? (((unsigned)(img * a.H) + (hp1 - 2u)) * (unsigned)a.W + (wp - 1u)) * (unsigned)(a.C * 2) : W_OOB;
    }
    if (tid < NT * 32) {   // output row of position p of the tile
        const int p = tid;
        const unsigned pr = (unsigned)(((unsigned long long)(unsigned)p * a.magic_pw) >> 40), pc = (unsigned)p - pr * (unsigned)a.PW;
        const int row = r0 + (int)pr, col = (int)pc - 1;
        const bool ok = (int)pr < a.rows_per_tile && row < a.H && (unsigned)col < (unsigned)a.W;
        out_tab[p] = ok ? (unsigned)((img * a.H + row) * a.W + col) * (unsigned)(a.Co * 2) : W_OOB;
    }
    lds_barrier();   // the tables
    {
        const int nvec = a.n_stage * 8;
        u32x4 st[W_LD0];
#pragma unroll
        for (int i = 0; i < W_LD0; ++i)
            if (i * W_THREADS < nvec) {
                const int v = tid + W_THREADS * i;   // v / 8 < W_TAB: the table ends with out-of-range entries
                st[i] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, in_tab[v >> 3] + (unsigned)((v & 7) * 16), 0, 0);
            }
#pragma unroll
        for (int i = 0; i < W_LD0; ++i)
            if (i * W_THREADS < nvec) {
                const int v = tid + W_THREADS * i;
                if (v < nvec) *(u32x4 *)(in_lds + (v >> 3) * a.row_bytes + (v & 7) * 16) = st[i];
            }
    }
    lds_barrier();   // group 0 is staged

    if (wave == 4) {
        __builtin_amdgcn_s_setprio(3);   // its few instructions should not queue behind the MFMAs of the wavefront it shares a SIMD with
        const unsigned lds_w0 = (unsigned)((lane >> 3) * a.row_bytes + (lane & 7) * 16);
        for (int g = 1; g < cpt; ++g) {
            for (int s0 = 0; s0 < a.n_stage; s0 += 8 * W_MAXLD) {
                u32x4 st[W_MAXLD];
#pragma unroll
                for (int i = 0; i < W_MAXLD; ++i)   // s0 + 7 + 8*35 < W_TAB
                    st[i] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, in_tab[s0 + (lane >> 3) + 8 * i] + (unsigned)(g * 128 + (lane & 7) * 16), 0, 0);
#pragma unroll
                for (int i = 0; i < W_MAXLD; ++i)
                    if (s0 + (lane >> 3) + 8 * i < a.n_stage) *(u32x4 *)(in_lds + lds_w0 + (unsigned)((s0 + 8 * i) * a.row_bytes + g * 128)) = st[i];
            }
            lds_barrier();   // group g is staged
        }
        __syncthreads();     // matches the barrier before the epilogue
        return;
    }

    // ---- accumulators: acc[p][4g+j] is channel 8g + 4*fk + j (of the wavefront's 32) at position 32p + frow
    f32x16 acc[NT];
    const int wcol0 = n0 + wave * 32;
    if (ACCUM) {
#pragma unroll
        for (int p = 0; p < NT; ++p) {
            const unsigned off = out_tab[p * 32 + frow];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int col = wcol0 + g * 8 + fk * 4;
                const u32x2 old = __builtin_amdgcn_raw_buffer_load_b64(out_rsrc, off != W_OOB ? off + (unsigned)(col * 2) : W_OOB, 0, 0);
                const bf16x4 ob = __builtin_bit_cast(bf16x4, old);
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[p][g * 4 + j] = (float)ob[j];
            }
        }
    } else {
#pragma unroll
        for (int p = 0; p < NT; ++p)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[p][v] = 0.f;
    }

    // ---- main loop over (64-channel group, tap).  The pixel fragments of k-step s+1 are read one by one behind the
    // MFMAs of k-step s; the last k-step of a tap already reads the next tap's first fragments.
    const unsigned lane_base = (unsigned)(frow * a.row_bytes + fk * 64);
    unsigned bp[NT];
    bf16x8 pf[2][NT];
    for (int g = 0; g < cpt; ++g) {
        if (g > 0) lds_barrier();   // group g is staged
        {
            const unsigned b0 = lane_base + (unsigned)(a.tapbyte[0] + g * 128);
#pragma unroll
            for (int p = 0; p < NT; ++p) {
                bp[p] = b0 + (unsigned)p * tile_step;
                pf[0][p] = *(const bf16x8 *)(in_lds + bp[p]);
            }
        }
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const unsigned to_next = t < 8 ? (unsigned)(a.tapbyte[t < 8 ? t + 1 : 0] - a.tapbyte[t]) : 0u;   // wraps for negative steps
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const bf16x8 wfrag = __builtin_bit_cast(bf16x8, wf[t % 3][s]);
#pragma unroll
                for (int p = 0; p < NT; ++p) {
                    acc[p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfrag, pf[s & 1][p], acc[p], 0, 0, 0);
                    if (s < 3) {
                        pf[(s + 1) & 1][p] = *(const bf16x8 *)(in_lds + bp[p] + (s + 1) * 16);
                    } else if (t < 8) {
                        bp[p] += to_next;
                        pf[0][p] = *(const bf16x8 *)(in_lds + bp[p]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            load_w(wf[t % 3]);
        }
    }
    __syncthreads();   // every wavefront is done with the staged input: it becomes the epilogue staging area

    // ---- epilogue: round to bf16, transpose one 32x32 accumulator at a time through this wavefront's strip, store
    // 16 contiguous bytes per lane (64 bytes per position and wavefront)
    constexpr int SROW = 80;   // 32 channels bf16 + 16 pad
    unsigned char *my_st = smem + wave * (32 * SROW);
    float ssum[8], ssq[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) ssum[e] = ssq[e] = 0.f;
    // out_tab lies behind the staged input, the strips at its start: no overlap as long as n_stage*row_bytes >= 4*32*80
#pragma unroll
    for (int p = 0; p < NT; ++p) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            bf16x4 pk;
#pragma unroll
            for (int j = 0; j < 4; ++j) pk[j] = (bf16_t)acc[p][g * 4 + j];
            *(bf16x4 *)(my_st + frow * SROW + (g * 8 + fk * 4) * 2) = pk;
        }
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const int idx = lane + 64 * jj, pos = idx >> 2, ck = idx & 3;
            const u32x4 v = *(const u32x4 *)(my_st + pos * SROW + ck * 16);
            const unsigned off = out_tab[p * 32 + pos];
            const bool live = off != W_OOB;
            __builtin_amdgcn_raw_buffer_store_b128(v, out_rsrc, live ? off + (unsigned)((wcol0 + ck * 8) * 2) : W_OOB, 0, 0);
            if (a.stats && live) {
                const bf16x8 vb = __builtin_bit_cast(bf16x8, v);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float f = (float)vb[e];
                    ssum[e] += f;
                    ssq[e] += f * f;
                }
            }
        }
    }
    if (a.stats) {
        // lanes with the same lane % 4 hold the same 8 channels
#pragma unroll
        for (int e = 0; e < 8; ++e)
#pragma unroll
            for (int o = 4; o < 64; o <<= 1) {
                ssum[e] += __shfl_xor(ssum[e], o, 64);
                ssq[e] += __shfl_xor(ssq[e], o, 64);
            }
        if (lane < 4) {
            float *r0p = a.stats + (size_t)tile * a.K + wcol0 + lane * 8;
            float *r1p = r0p + (size_t)a.stats_rows * a.K;
            *(f32x4 *)r0p = f32x4{ssum[0], ssum[1], ssum[2], ssum[3]};
            *(f32x4 *)(r0p + 4) = f32x4{ssum[4], ssum[5], ssum[6], ssum[7]};
            *(f32x4 *)r1p = f32x4{ssq[0], ssq[1], ssq[2], ssq[3]};
            *(f32x4 *)(r1p + 4) = f32x4{ssq[4], ssq[5], ssq[6], ssq[7]};
        }
    }
}

constexpr int kNT = 7;   // position tiles per block of the one instance built

struct Plan {
    int rows_per_tile, tiles_per_img, n_stage, row_bytes, smem;
};

bool make_plan(const IgemmArgs &g, Plan *p)
{
    const int PW = g.Ws + 2;
    if (PW > kNT * 32) return false;
    p->rows_per_tile = kNT * 32 / PW;
    if (p->rows_per_tile > g.Hs) p->rows_per_tile = g.Hs;
    p->tiles_per_img = ceil_div(g.Hs, p->rows_per_tile);
    p->n_stage = kNT * 32 + 2 * (PW + 1);
    p->row_bytes = g.Cs * 2 + 16;
    p->smem = p->n_stage * p->row_bytes + (kNT * 32 + W_TAB) * 4;
    return p->smem <= W_LDS_MAX && p->n_stage <= W_STAGE_MAX;
}

}  // namespace

bool halo_wide_applicable(int dtype, const IgemmArgs &a)
{
    if (dtype != NSK_BF16 || getenv("NSK_NO_HALO_WIDE") != nullptr) return false;
    if (a.ntaps != 9 || (a.Cs != 128 && a.Cs != 256 && a.Cs != 512) || a.Ngemm % W_BN != 0 || a.Co % 8 != 0) return false;
    if (a.Ktot != 9 * a.Cs) return false;
    if (a.mult_h != 1 || a.mult_w != 1 || a.osh != 1 || a.osw != 1 || a.oa != 0 || a.ob != 0) return false;
    if (a.Hs != a.Ho || a.Ws != a.Wo || a.Mi != a.Ho || a.Mj != a.Wo) return false;
    for (int t = 0; t < 9; ++t) {
        const int eh = a.add_h + a.off_h[t], ew = a.add_w + a.off_w[t];
        if (eh < -1 || eh > 1 || ew < -1 || ew > 1) return false;
    }
    Plan p;
    if (!make_plan(a, &p)) return false;
    const long long out_bytes = (long long)a.Nimg * a.Ho * a.Wo * a.Co * 2;
    if ((unsigned long long)a.src_bytes >= W_OOB || (unsigned long long)a.wpk_bytes >= W_OOB || out_bytes >= (long long)W_OOB) return false;
    if (((uintptr_t)a.src | (uintptr_t)a.wpk | (uintptr_t)a.out) & 15) return false;
    // the positions a tile computes beyond the image rows it owns are wasted MFMA work: take the layer only if at
    // least two thirds of it is useful, and only if the tiles fill a good part of the chip (NSK_HALO_WIDE_ALWAYS:
    // test hook, small shapes)
    if (getenv("NSK_HALO_WIDE_ALWAYS") != nullptr) return true;
    const long long useful = (long long)a.Hs * a.Ws, computed = (long long)p.tiles_per_img * kNT * 32;
    if (useful * 3 < computed * 2) return false;
    return (long long)a.Nimg * p.tiles_per_img * (a.Ngemm / W_BN) >= 128;
}

int halo_wide_stats_rows(const IgemmArgs &a)
{
    Plan p;
    if (a.accumulate || !make_plan(a, &p)) return 0;
    return a.Nimg * p.tiles_per_img;
}

int launch_halo_wide(const IgemmArgs &g, hipStream_t stream)
{
    Plan p;
    if (!make_plan(g, &p)) return NSK_ERR_BAD_DESC;
    WideArgs a{};
    a.src = g.src; a.wpk = g.wpk; a.out = g.out;
    a.N = g.Nimg; a.H = g.Hs; a.W = g.Ws; a.C = g.Cs; a.K = g.Ngemm; a.Co = g.Co;
    a.PW = g.Ws + 2;
    a.rows_per_tile = p.rows_per_tile;
    a.tiles_per_img = p.tiles_per_img;
    a.tiles = g.Nimg * p.tiles_per_img;
    a.n_stage = p.n_stage;
    a.row_bytes = p.row_bytes;
    a.magic_pw = ((1ULL << 40) + a.PW - 1) / a.PW;
    a.src_bytes = g.src_bytes; a.wpk_bytes = g.wpk_bytes;
    a.out_bytes = (unsigned)((long long)g.Nimg * g.Ho * g.Wo * g.Co * 2);
    a.accumulate = g.accumulate;
    for (int t = 0; t < 9; ++t)
        a.tapbyte[t] = (a.PW + 1 + (g.add_h + g.off_h[t]) * a.PW + (g.add_w + g.off_w[t])) * a.row_bytes;
    a.stats = g.stats; a.stats_rows = g.stats_rows;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)conv_halo_wide_kernel<kNT, false>, hipFuncAttributeMaxDynamicSharedMemorySize, W_LDS_MAX);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)conv_halo_wide_kernel<kNT, true>, hipFuncAttributeMaxDynamicSharedMemorySize, W_LDS_MAX);
        if (e != hipSuccess) {
            set_last_hip_error(e);
            return NSK_ERR_HIP;
        }
        attr_set = true;
    }
    const dim3 grid((unsigned)(a.tiles * (a.K / W_BN)));
    if (g.accumulate)
        hipLaunchKernelGGL((conv_halo_wide_kernel<kNT, true>), grid, dim3(W_THREADS), p.smem, stream, a);
    else
        hipLaunchKernelGGL((conv_halo_wide_kernel<kNT, false>), grid, dim3(W_THREADS), p.smem, stream, a);
    return check_launch();
}

}  // namespace nsk

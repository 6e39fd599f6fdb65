// 3x3 bf16 convolution with 64, 128 or 256 input channels and a multiple of 64 output channels: forward and backward-data of
// stride-1 layers, and backward-data of strided layers (whose residue classes are stride-1 convolutions over dy).
// These are the 3x3 layers of the later bottleneck stages of the residual networks the paper trains (section
// "Experiments and Discussion"); with 2304 or more reduction indices they are the layers where the matrix units, not
// memory, should be the limit.
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
//     a time by an extra wavefront, group g+1 while group g is multiplied, so only the first group's loads are exposed
//     (one barrier per group).
// Block = NT*32 positions x 128 (or 64) output channels, 4 (or 2) multiplying wavefronts + 1 that moves data; wavefront w owns channels 32w..32w+31 of all NT position
// tiles (NT accumulators of 32x32).  For 14 x 14 images a tile is exactly one image (14 rows of 16 padded positions).
#include <stdlib.h>

#include "nsk_internal.h"

namespace nsk {
namespace {

constexpr unsigned W_OOB = 0xF0000000u;
constexpr int W_LDS_MAX = 160 * 1024;               // epilogue strips + staged input + tables
constexpr int W_MAXLD = 36;                         // 16-byte loads the moving wavefront keeps in flight
constexpr int W_STAGE_MAX = 576;                    // staged positions of a tile, at most (two rounds of the moving wavefront)
constexpr int W_TAB = 640;                          // entries of the staged-position table (two per thread)

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) const bf16x8 lds_bf16x8;

// 16-byte LDS read at a 32-bit LDS address (no generic-pointer arithmetic: the address register goes straight into
// the instruction, constants into its offset field)
__device__ __forceinline__ bf16x8 lds_read16(unsigned addr)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return *(lds_bf16x8 *)addr;
#else
    return bf16x8{};   // the host pass only parses this (its pointers are 64 bits wide)
#endif
}

constexpr int W_CLS = 4;     // output classes of one launch

// One launch = up to four "classes" that read the same source tensor through the same tiles and write disjoint
// position sets of the same output tensor: the forward pass and the backward-data pass of a stride-1 layer have one
// class with nine taps; the backward-data pass of a stride-2 3x3 layer has four (the residue classes of the output
// position modulo 2, with 4, 2, 2 and 1 taps), each a stride-1 convolution over the same dy tile.
struct WideArgs {
    const void *src;
    void *out;
    const void *wpk[W_CLS];       // packed filter of each class: [K][ntaps][C]
    unsigned wpk_bytes[W_CLS];
    int ntaps[W_CLS];
    int Mi[W_CLS], Mj[W_CLS];     // output extent of each class in tile coordinates
    int oa[W_CLS], ob[W_CLS];     // output position of (i, j): (i*osh + oa, j*osw + ob)
    unsigned long long tapcode[W_CLS];   // 4 bits per tap: (dh + 1) * 4 + (dw + 1)
    int ncls;
    int N, H, W, C, K;            // source extent, channels in, channels out
    int Ho, Wo, Co, osh, osw;
    int PW;                       // padded width W + 2
    int rows_per_tile, tiles_per_img, tiles;
    int n_stage;                  // staged positions: NT*32 + 2*(PW + 1)
    int row_bytes;                // LDS bytes per staged position: 2*C + 16
    unsigned magic_pw;            // ceil(2^32 / PW): u / PW = mulhi(u, magic_pw) for u * PW < 2^32
    unsigned src_bytes, out_bytes;
    float *stats;                 // single class only: per-channel partial sums of the stored output (one row per tile)
    int stats_rows;
    // MERGE launches (the forward pass of a stride-2 layer): the classes are the four parity planes of the input,
    // plane (pa, pb) = x[2I-1+pa][2J-1+pb] on the output's own grid, each with the taps that fall on it (shifts 0 or +1);
    // they are staged one after the other, add into ONE set of accumulators and share one epilogue.  The filter is
    // the forward filter itself ([K][wrow_taps][C]); tapidx holds, 4 bits per tap of a class, the tap's place in it.
    int pa[W_CLS], pb[W_CLS];
    unsigned long long tapidx[W_CLS];
    int wrow_taps;
    int Hx, Wx;                   // extent of x
};

template <typename T> __device__ __forceinline__ T sel4(const T (&v)[W_CLS], int c)
{
    return c == 0 ? v[0] : c == 1 ? v[1] : c == 2 ? v[2] : v[3];
}

// MW multiplying wavefronts (32 output channels each) and one that moves data; at most two wavefronts per SIMD, so
// that two of the smaller blocks (MW = 2, 64 output channels) share a CU.
// MODE: 0 plain, 1 accumulate into the old output, 2 plain with the statistics epilogue (single class).
// NINE: a single class with nine taps, tap loop unrolled.
// MERGE: see WideArgs.  The input of such a launch is four times that of a stride-1 layer for the same MFMA count, in
// sixteen stages (plane, 64-channel group) of which the shortest is multiplied in 900 clocks: TWO wavefronts move data,
// each half of a stage's rows, with the requests running two stages ahead of the LDS writes.
template <int NT, int MW, int MODE, bool NINE, bool MERGE = false>
__global__ __launch_bounds__((MW + (MERGE ? 2 : 1)) * 64) __attribute__((amdgpu_waves_per_eu(2))) void conv_halo_wide_kernel(const WideArgs a)
{
    static_assert(!(MERGE && (NINE || MODE == 1)), "merged planes: the generic piece loop, no accumulation into old outputs");
    constexpr int THREADS = (MW + (MERGE ? 2 : 1)) * 64, BN = MW * 32;
    constexpr bool ACCUM = MODE == 1, STATS = MODE == 2;
    constexpr int LD0 = (W_STAGE_MAX * 8 + THREADS - 1) / THREADS;   // loads per thread for the first group
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int SROW = 80, STRIP = 32 * SROW;                        // epilogue strip: 32 rows of 32 channels bf16 + 16 pad
    unsigned char *strips = smem;                                       // two per multiplying wavefront
    unsigned char *in_lds = smem + MW * 2 * STRIP;
    // per position of the tile: byte offset of output position (row*osh, col*osw) (a class adds its own shift), and
    // (row << 16 | col) in tile-grid coordinates, 0xFFFFFFFF for positions that are no output at all
    unsigned *out_tab = (unsigned *)(in_lds + a.n_stage * a.row_bytes);
    unsigned *rc_tab = out_tab + NT * 32;
    unsigned *in_tab = rc_tab + NT * 32;                                // W_TAB byte offsets of the staged positions

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int frow = lane & 31, fk = lane >> 5;

    // block id -> (tile, column block).  Consecutive ids run on different XCDs; with two column blocks an XCD sees
    // only one half of the filter.
    const int tiles_n = a.K / BN;
    const int nt = (int)blockIdx.x % tiles_n, tile = (int)blockIdx.x / tiles_n;
    const int img = tile / a.tiles_per_img, r0 = (tile - img * a.tiles_per_img) * a.rows_per_tile;
    const int n0 = nt * BN;

    const __amdgpu_buffer_rsrc_t src_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.src, 0, a.src_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t out_rsrc = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, a.out_bytes, 0x00020000);

    const int cpt = a.C >> 6;    // 64-channel groups
    const unsigned tile_step = (unsigned)(32 * a.row_bytes);

    // ---- filter stream (wavefronts 0..3).  The reduction runs over "pieces": one (class, 64-channel group, tap),
    // classes outermost, taps innermost.  Lane (row r = lane % 32, half h = lane / 32) reads bytes [64h, 64h + 64) of
    // the 128 bytes a piece occupies in filter row n0 + 32*wave + r of its class.  Three pieces are in flight; the
    // first three of a class are requested before the epilogue of the class before it.
    const unsigned wrow_idx = (unsigned)(n0 + (wave < MW ? wave : 0) * 32 + frow);
    u32x4 wf[3][4];
    // per class: filter descriptor, taps, byte offset of the lane's row; (tap, group) of the next piece to load
    __amdgpu_buffer_rsrc_t w_rs;
    int w_ntaps = 1, ld_t = 0, ld_g = 0;
    unsigned w_row = 0;
    unsigned long long w_tapidx = 0;
    auto filter_class = [&](int c) {
        w_ntaps = sel4(a.ntaps, c);
        w_rs = __builtin_amdgcn_make_buffer_rsrc((void *)sel4(a.wpk, c), 0, sel4(a.wpk_bytes, c), 0x00020000);
        w_row = wrow_idx * (unsigned)((MERGE ? a.wrow_taps : w_ntaps) * a.C * 2) + (unsigned)(fk * 64);
        if (MERGE) w_tapidx = sel4(a.tapidx, c);
        ld_t = 0;
        ld_g = 0;
    };
    // byte offset of tap t of the class inside a filter row
    auto tap_bytes = [&](int t) -> unsigned { return (unsigned)((MERGE ? (int)(w_tapidx >> (4 * t)) & 15 : t) * a.C * 2); };
    auto load_w = [&](u32x4 (&Wf)[4]) {   // past the last piece of the class: nothing (zeros)
        const unsigned off = ld_g < cpt ? w_row + tap_bytes(ld_t) + (unsigned)(ld_g * 128) : W_OOB;
#pragma unroll
        for (int s = 0; s < 4; ++s) Wf[s] = __builtin_amdgcn_raw_buffer_load_b128(w_rs, off + (unsigned)(s * 16), 0, 0);
        if (++ld_t >= w_ntaps) {
            ld_t = 0;
            ++ld_g;
        }
    };
    filter_class(0);
    if (wave < MW) {   // (the moving wavefronts have no filter rows)
        load_w(wf[0]);
        load_w(wf[1]);
        load_w(wf[2]);
    }

    // ---- staging.  Staged position s is position r0*PW - 1 + s of the zero-padded image (row-major from the top-left
    // corner of the padding); in_tab[s] is its byte offset in src, or out of range for padding.  The tile is staged
    // one 64-channel group at a time: group 0 by all wavefronts, group g+1 by the last wavefront alone while the
    // others multiply group g of the first class (they meet at one barrier per group).  After the first group no
    // input load is exposed, and the multiplying wavefronts have nothing but their filter stream in their (in-order)
    // load queue.  One-time code is kept short on purpose: a block runs once per launch, so all of it is fetched cold.
    // byte offset in src of staged position s (of plane c with merged planes), out of range for padding
    auto stage_offset = [&](int s, int c) -> unsigned {
        // u counts from one row above the padded image (so that it is never negative): u / PW is the image row + 2,
        // u % PW the image column + 1
        const unsigned u = (unsigned)((r0 + 1) * a.PW - 1 + s);
        const unsigned hp1 = __umulhi(u, a.magic_pw);
        const unsigned wp = u - hp1 * (unsigned)a.PW;
        if (MERGE) {   // grid position (I, J) = (hp1 - 2, wp - 1) of plane c is pixel (2I - 1 + pa, 2J - 1 + pb) of x
            const unsigned h = 2u * (hp1 - 2u) - 1u + (unsigned)sel4(a.pa, c), w = 2u * (wp - 1u) - 1u + (unsigned)sel4(a.pb, c);
            const bool ok = s < a.n_stage && h < (unsigned)a.Hx && w < (unsigned)a.Wx;
            return ok ? (((unsigned)(img * a.Hx) + h) * (unsigned)a.Wx + w) * (unsigned)(a.C * 2) : W_OOB;
        }
        const bool ok = s < a.n_stage && (hp1 - 2u < (unsigned)a.H) && (wp - 1u < (unsigned)a.W);
        return ok ? (((unsigned)(img * a.H) + (hp1 - 2u)) * (unsigned)a.W + (wp - 1u)) * (unsigned)(a.C * 2) : W_OOB;
    };
    for (int s = tid; s < W_TAB; s += THREADS) in_tab[s] = stage_offset(s, 0);
    for (unsigned p = (unsigned)tid; p < (unsigned)(NT * 32); p += THREADS) {   // (fewer threads than positions when MW = 2)
        const unsigned pr = __umulhi(p, a.magic_pw), pc = p - pr * (unsigned)a.PW;
        const int row = r0 + (int)pr, col = (int)pc - 1;
        const bool ok = (int)pr < a.rows_per_tile && row < a.H && (unsigned)col < (unsigned)a.W;
        out_tab[p] = (unsigned)((img * a.Ho + row * a.osh) * a.Wo + col * a.osw) * (unsigned)(a.Co * 2);
        rc_tab[p] = ok ? (unsigned)row << 16 | (unsigned)col : 0xFFFFFFFFu;
    }
    lds_barrier();   // the tables
    {
        const int nvec = a.n_stage * 8;
        u32x4 st[LD0];
#pragma unroll
        for (int i = 0; i < LD0; ++i)
            if (i * THREADS < nvec) {
                const int v = tid + THREADS * i;   // v / 8 < W_TAB: the table ends with out-of-range entries
                st[i] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, in_tab[v >> 3] + (unsigned)((v & 7) * 16), 0, 0);
            }
#pragma unroll
        for (int i = 0; i < LD0; ++i)
            if (i * THREADS < nvec) {
                const int v = tid + THREADS * i;
                if (v < nvec) *(u32x4 *)(in_lds + (v >> 3) * a.row_bytes + (v & 7) * 16) = st[i];
            }
    }
    lds_barrier();   // group 0 is staged

    if (MERGE && wave >= MW) {
        __builtin_amdgcn_s_setprio(3);
        // Stage k = (plane k / cpt, group k % cpt), k = 1 .. 4*cpt - 1, is written to LDS while stage k - 1 is multiplied
        // (its columns were last read a whole plane, or two stages, ago) and was requested two stages earlier.  This
        // wavefront owns rows [m*HALF, m*HALF + HALF) of every stage: row (lane / 8) + 8*i of them in load i, 16 bytes per
        // lane.  The byte offset of a row is computed once per plane, by lane r % 64 for row r (register r / 64), and
        // reaches the eight lanes that load the row through a lane exchange.
        constexpr int NL = 18, HALF = 8 * NL;          // n_stage <= 2 * HALF (the launcher checks)
        const int m = wave - MW;
        const unsigned lds_w0 = (unsigned)((m * HALF + (lane >> 3)) * a.row_bytes + (lane & 7) * 16);
        const int stages = a.ncls * cpt;
        unsigned mine[3];
        int mine_cls = -1;
        u32x4 stA[NL], stB[NL];
        auto request = [&](int k, u32x4 (&st)[NL]) {
            if (k >= stages) return;
            const int c = k / cpt, g = k & (cpt - 1);   // cpt is 2 or 4
            if (c != mine_cls) {
#pragma unroll
                for (int q = 0; q < 3; ++q) mine[q] = stage_offset(m * HALF + 64 * q + lane, c);
                mine_cls = c;
            }
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const unsigned off = (unsigned)__builtin_amdgcn_ds_bpermute(((lane >> 3) + 8 * (i & 7)) * 4, (int)mine[i >> 3]);
                st[i] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, off + (unsigned)(g * 128 + (lane & 7) * 16), 0, 0);
            }
        };
        auto commit = [&](int k, const u32x4 (&st)[NL]) {
            const int g = k & (cpt - 1);
#pragma unroll
            for (int i = 0; i < NL; ++i)
                if (m * HALF + (lane >> 3) + 8 * i < a.n_stage) *(u32x4 *)(in_lds + lds_w0 + (unsigned)(8 * i * a.row_bytes + g * 128)) = st[i];
        };
        request(1, stA);
        request(2, stB);
        for (int k = 1; k < stages; k += 2) {
            commit(k, stA);
            request(k + 2, stA);
            lds_barrier();   // stage k is in place
            if (k + 1 >= stages) break;
            commit(k + 1, stB);
            request(k + 3, stB);
            lds_barrier();   // stage k + 1 is in place
        }
        return;
    }
    if (!MERGE && wave == MW) {
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
        return;
    }

    // ---- accumulators: acc[p][4g+j] is channel 8g + 4*fk + j (of the wavefront's 32) at position 32p + frow
    f32x16 acc[NT];
    const int wcol0 = n0 + wave * 32;
    // byte offset of channel wcol0 + 8*ck at position `pos` of the tile in class `cls`, or out of range where the class
    // has no output
    auto out_offset = [&](unsigned shift, unsigned mi, unsigned mj, int pos, int ck) -> unsigned {
        const unsigned rc = rc_tab[pos];
        const unsigned off = out_tab[pos];
        return ((rc >> 16) < mi && (rc & 0xFFFFu) < mj) ? off + shift + (unsigned)((wcol0 + ck * 8) * 2) : W_OOB;   // 0xFFFF fails the row test
    };
    auto init_acc = [&](int cls) {
        if (ACCUM) {   // start from the old values: the sum is rounded to bf16 exactly once
            const unsigned shift = (unsigned)((sel4(a.oa, cls) * a.Wo + sel4(a.ob, cls)) * a.Co * 2);
            const unsigned mi = (unsigned)sel4(a.Mi, cls), mj = (unsigned)sel4(a.Mj, cls);
#pragma unroll
            for (int p = 0; p < NT; ++p) {
                const unsigned off = out_offset(shift, mi, mj, p * 32 + frow, 0);
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const u32x2 old = __builtin_amdgcn_raw_buffer_load_b64(out_rsrc, off != W_OOB ? off + (unsigned)((g * 8 + fk * 4) * 2) : W_OOB, 0, 0);
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
    };

    // ---- epilogue of one class: round to bf16, transpose one 32x32 accumulator at a time through one of this
    // wavefront's two strips (tile p+1 is written while tile p is read back), store 16 contiguous bytes per lane (64
    // bytes per position and wavefront).  Stores of 8 bytes per lane straight from the accumulators need no LDS but
    // took 2.5 times as long.
    unsigned char *my_st = strips + wave * (2 * STRIP);
    auto epilogue = [&](int cls) {
        const unsigned shift = (unsigned)((sel4(a.oa, cls) * a.Wo + sel4(a.ob, cls)) * a.Co * 2);
        const unsigned mi = (unsigned)sel4(a.Mi, cls), mj = (unsigned)sel4(a.Mj, cls);
        float ssum[8], ssq[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) ssum[e] = ssq[e] = 0.f;
        auto to_strip = [&](int p) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                bf16x4 pk;
#pragma unroll
                for (int j = 0; j < 4; ++j) pk[j] = (bf16_t)acc[p][g * 4 + j];
                *(bf16x4 *)(my_st + (p & 1) * STRIP + frow * SROW + (g * 8 + fk * 4) * 2) = pk;
            }
        };
        // tile p's rows are read back (and their output offsets looked up) before tile p+1 is converted and written to
        // the other strip, and stored after it: the LDS round trip hides behind the conversion
        u32x4 v[2][2];
        unsigned off[2][2];
        auto read_back = [&](int p) {
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
                const int idx = lane + 64 * jj, pos = idx >> 2, ck = idx & 3;
                off[p & 1][jj] = out_offset(shift, mi, mj, p * 32 + pos, ck);
                v[p & 1][jj] = *(const u32x4 *)(my_st + (p & 1) * STRIP + pos * SROW + ck * 16);
            }
        };
        to_strip(0);
        read_back(0);
#pragma unroll
        for (int p = 0; p < NT; ++p) {
            if (p + 1 < NT) to_strip(p + 1);
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
                __builtin_amdgcn_raw_buffer_store_b128(v[p & 1][jj], out_rsrc, off[p & 1][jj], 0, 0);
                if (STATS && off[p & 1][jj] != W_OOB) {
                    const bf16x8 vb = __builtin_bit_cast(bf16x8, v[p & 1][jj]);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float f = (float)vb[e];
                        ssum[e] += f;
                        ssq[e] += f * f;
                    }
                }
            }
            if (p + 1 < NT) read_back(p + 1);
        }
        if (STATS) {
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
    };

    // ---- main loop over the pieces.  The pixel fragments of k-step s+1 are read one by one behind the MFMAs of k-step
    // s; the last k-step of a piece already reads the next piece's first fragments, unless that piece opens a group
    // that is still being staged (first class only: then they are read after the barrier) or a new class.
    // lane 16*c + t keeps the LDS shift of tap t = (dh, dw) of class c: (PW + 1 + dh*PW + dw) * row_bytes
    const int my_code = (int)(sel4(a.tapcode, lane >> 4) >> (4 * (lane & 15))) & 15;
    const int my_tap = (a.PW + 1 + ((my_code >> 2) - 1) * a.PW + ((my_code & 3) - 1)) * a.row_bytes;
    const unsigned lane_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)in_lds + (unsigned)(frow * a.row_bytes + fk * 64);
    unsigned bp[NT];
    bf16x8 pf[2][NT];
    int cls = 0, tap = 0, grp = 0;      // the piece being multiplied
    int ntaps_c = a.ntaps[0];
    auto first_fragments = [&]() {
        const unsigned b0 = lane_base + (unsigned)(__builtin_amdgcn_readlane(my_tap, 16 * cls + tap) + grp * 128);
#pragma unroll
        for (int p = 0; p < NT; ++p) {
            bp[p] = b0 + (unsigned)p * tile_step;
            asm volatile("" : "+v"(bp[p]));
            pf[0][p] = lds_read16(bp[p]);
        }
    };
    init_acc(0);
    first_fragments();
    // The bookkeeping of a piece (which piece follows, where its fragments and the next filter piece lie) is spread
    // over the gaps between its first MFMAs: a wavefront issues in order, and fifty scalar instructions between two
    // pieces would cost several MFMA slots.
    auto piece = [&](u32x4 (&Wf)[4]) {
        int tn = 0, gn = 0;
        bool wait_group = false;
        unsigned to_next = 0u, w_off = W_OOB;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const bf16x8 wfrag = __builtin_bit_cast(bf16x8, Wf[s]);
#pragma unroll
            for (int p = 0; p < NT; ++p) {
                acc[p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfrag, pf[s & 1][p], acc[p], 0, 0, 0);
                if (s < 3) {
                    pf[(s + 1) & 1][p] = lds_read16(bp[p] + (s + 1) * 16);
                } else {
                    bp[p] += to_next;
                    asm volatile("" : "+v"(bp[p]));   // keep the running address in its register (else: base + scalar sum, one add per read)
                    pf[0][p] = lds_read16(bp[p]);
                }
                if (s == 0 && p == 0) {   // the piece after this one
                    tn = tap + 1;
                    gn = grp;
                    if (tn == ntaps_c) {
                        tn = 0;
                        ++gn;
                    }
                }
                if (s == 0 && p == 1) {
                    const bool class_ends = gn == cpt;
                    wait_group = !class_ends && tn == 0 && cls == 0;   // group gn of the first class: staged behind a barrier
                    // without a piece to read ahead the fragments are re-read where they are: in range, unused
                    if (!class_ends && !wait_group)
                        to_next = (unsigned)(__builtin_amdgcn_readlane(my_tap, 16 * cls + tn) + gn * 128) -
                                  (unsigned)(__builtin_amdgcn_readlane(my_tap, 16 * cls + tap) + grp * 128);   // wraps for negative steps
                }
                if (s == 0 && p == 2) {   // the filter piece to request into this set: three pieces ahead
                    if (ld_g < cpt) w_off = w_row + tap_bytes(ld_t) + (unsigned)(ld_g * 128);
                    if (++ld_t >= w_ntaps) {
                        ld_t = 0;
                        ++ld_g;
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            // this k-step's filter fragment is spent
            Wf[s] = __builtin_amdgcn_raw_buffer_load_b128(w_rs, w_off + (unsigned)(s * 16), 0, 0);
        }
        tap = tn;
        grp = gn;
        if (wait_group) {
            lds_barrier();   // group gn is staged
            first_fragments();
        }
    };
    // Merged planes: the pieces of all planes are ONE sequence (plane, group, tap), so the filter stream runs through
    // the plane changes without a restart; every stage (plane, group) but the first waits for its barrier.
    if (MERGE) {
        int ld_c = 0;   // plane of the next filter piece to request
        auto piece_m = [&](u32x4 (&Wf)[4]) {
            int tn = 0, gn = 0, cn = 0;
            bool wait_stage = false;
            unsigned to_next = 0u, w_off = W_OOB;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const bf16x8 wfrag = __builtin_bit_cast(bf16x8, Wf[s]);
#pragma unroll
                for (int p = 0; p < NT; ++p) {
                    acc[p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfrag, pf[s & 1][p], acc[p], 0, 0, 0);
                    if (s < 3) {
                        pf[(s + 1) & 1][p] = lds_read16(bp[p] + (s + 1) * 16);
                    } else {
                        bp[p] += to_next;
                        asm volatile("" : "+v"(bp[p]));
                        pf[0][p] = lds_read16(bp[p]);
                    }
                    if (s == 0 && p == 0) {   // the piece after this one
                        tn = tap + 1;
                        gn = grp;
                        cn = cls;
                        if (tn == ntaps_c) {
                            tn = 0;
                            if (++gn == cpt) {
                                gn = 0;
                                ++cn;
                            }
                        }
                    }
                    if (s == 0 && p == 1) {
                        wait_stage = cn < a.ncls && tn == 0;   // a new stage: staged behind a barrier
                        if (cn < a.ncls && !wait_stage)        // the next tap of the same stage: read ahead
                            to_next = (unsigned)(__builtin_amdgcn_readlane(my_tap, 16 * cls + tn) - __builtin_amdgcn_readlane(my_tap, 16 * cls + tap));
                    }
                    if (s == 0 && p == 2) {   // the filter piece to request into this set: three pieces ahead
                        if (ld_c < a.ncls) w_off = w_row + tap_bytes(ld_t) + (unsigned)(ld_g * 128);
                        if (++ld_t >= w_ntaps) {
                            ld_t = 0;
                            if (++ld_g >= cpt) {
                                ld_g = 0;
                                if (++ld_c < a.ncls) {
                                    w_ntaps = sel4(a.ntaps, ld_c);
                                    w_tapidx = sel4(a.tapidx, ld_c);
                                }
                            }
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                Wf[s] = __builtin_amdgcn_raw_buffer_load_b128(w_rs, w_off + (unsigned)(s * 16), 0, 0);
            }
            tap = tn;
            grp = gn;
            if (cn != cls) {
                cls = cn;
                if (cls < a.ncls) ntaps_c = sel4(a.ntaps, cls);
            }
            if (wait_stage) {
                lds_barrier();   // the stage is in place
                first_fragments();
            }
        };
        const int total = 9 * cpt;   // a multiple of three
        for (int i = 0; i < total; i += 3) {
            piece_m(wf[0]);
            piece_m(wf[1]);
            piece_m(wf[2]);
        }
        epilogue(0);   // one output, described by every class alike
        return;
    }
    // A single class with nine taps (forward, backward-data at stride 1): the same pieces with the tap loop unrolled, so
    // that tap shifts are scalars known per call and a piece carries no bookkeeping at all (8% off the main loop).
    if (NINE) {
        int shift[9];
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const int code = (int)(a.tapcode[0] >> (4 * t)) & 15;
            shift[t] = (a.PW + 1 + ((code >> 2) - 1) * a.PW + ((code & 3) - 1)) * a.row_bytes;
        }
        for (int g = 0; g < cpt; ++g) {
            if (g > 0) {
                lds_barrier();   // group g is staged
                grp = g;
                first_fragments();
            }
#pragma unroll
            for (int t = 0; t < 9; ++t) {
                const unsigned to_next = t < 8 ? (unsigned)(shift[t + 1] - shift[t]) : 0u;   // last tap: re-read in place (unused)
                const unsigned w_off = ld_g < cpt ? w_row + (unsigned)(ld_t * a.C * 2 + ld_g * 128) : W_OOB;
                if (++ld_t == 9) {
                    ld_t = 0;
                    ++ld_g;
                }
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const bf16x8 wfrag = __builtin_bit_cast(bf16x8, wf[t % 3][s]);
#pragma unroll
                    for (int p = 0; p < NT; ++p) {
                        acc[p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfrag, pf[s & 1][p], acc[p], 0, 0, 0);
                        if (s < 3) {
                            pf[(s + 1) & 1][p] = lds_read16(bp[p] + (s + 1) * 16);
                        } else {
                            bp[p] += to_next;
                            asm volatile("" : "+v"(bp[p]));
                            pf[0][p] = lds_read16(bp[p]);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    wf[t % 3][s] = __builtin_amdgcn_raw_buffer_load_b128(w_rs, w_off + (unsigned)(s * 16), 0, 0);
                }
            }
        }
        epilogue(0);
        return;
    }
    if (!NINE && !MERGE)
    for (;;) {
        const int np = ntaps_c * cpt;
        int i = 0;
        for (; i + 3 <= np; i += 3) {
            piece(wf[0]);
            piece(wf[1]);
            piece(wf[2]);
        }
        if (i < np) piece(wf[0]);
        if (i + 1 < np) piece(wf[1]);
        const bool more = !STATS && cls + 1 < a.ncls;   // the statistics epilogue comes with a single class
        if (more) {   // the next class's filter is on its way while this one is stored
            filter_class(cls + 1);
            load_w(wf[0]);
            load_w(wf[1]);
            load_w(wf[2]);
        }
        epilogue(cls);
        if (!more) break;
        ++cls;
        tap = 0;
        grp = 0;
        ntaps_c = w_ntaps;
        init_acc(cls);
        first_fragments();
    }
}

constexpr int kNT = 7;   // position tiles per block of the one instance built

// 128 output channels per block where the layer has a multiple of that, else 64 (blocks of two multiplying wavefronts)
int block_channels(const IgemmArgs &g) { return g.Ngemm % 128 == 0 ? 128 : 64; }

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
    p->smem = block_channels(g) / 32 * 2 * 32 * 80 + p->n_stage * p->row_bytes + (2 * kNT * 32 + W_TAB) * 4;
    // (exactness of the reciprocal division of staged positions by PW; rows fit 16 bits)
    if (((long long)(g.Hs + 3) * PW + W_TAB) * PW >= (1LL << 32) || g.Hs >= 65535) return false;
    return p->smem <= W_LDS_MAX && p->n_stage <= W_STAGE_MAX;
}

// Shape tests of one class; `first` is the class the shared fields are compared with.
bool class_ok(const IgemmArgs &a, const IgemmArgs &first)
{
    if (a.ntaps < 1 || a.ntaps > 9 || (a.Cs != 64 && a.Cs != 128 && a.Cs != 256) || a.Ngemm % 64 != 0 || a.Co % 8 != 0) return false;
    if (a.Ktot != a.ntaps * a.Cs || a.stats_rows < 0) return false;
    if (a.mult_h != 1 || a.mult_w != 1 || a.Mi > a.Hs || a.Mj > a.Ws || a.Mi < 1 || a.Mj < 1) return false;
    if (a.osh < 1 || a.osw < 1 || a.oa < 0 || a.ob < 0) return false;
    if ((a.Mi - 1) * a.osh + a.oa >= a.Ho || (a.Mj - 1) * a.osw + a.ob >= a.Wo) return false;
    for (int t = 0; t < a.ntaps; ++t) {
        const int eh = a.add_h + a.off_h[t], ew = a.add_w + a.off_w[t];
        if (eh < -1 || eh > 1 || ew < -1 || ew > 1) return false;
    }
    if (a.src != first.src || a.out != first.out || a.Cs != first.Cs || a.Ngemm != first.Ngemm || a.Nimg != first.Nimg ||
        a.Hs != first.Hs || a.Ws != first.Ws || a.Ho != first.Ho || a.Wo != first.Wo || a.Co != first.Co || a.osh != first.osh ||
        a.osw != first.osw || a.accumulate != first.accumulate || a.src_bytes != first.src_bytes)
        return false;
    if ((unsigned long long)a.wpk_bytes >= W_OOB || ((uintptr_t)a.wpk & 15)) return false;
    return true;
}

bool classes_ok(const IgemmArgs *a, int count)
{
    if (count < 1 || count > W_CLS) return false;
    for (int i = 0; i < count; ++i)
        if (!class_ok(a[i], a[0])) return false;
    Plan p;
    if (!make_plan(a[0], &p)) return false;
    const long long out_bytes = (long long)a[0].Nimg * a[0].Ho * a[0].Wo * a[0].Co * 2;
    if ((unsigned long long)a[0].src_bytes >= W_OOB || out_bytes >= (long long)W_OOB) return false;
    if (((uintptr_t)a[0].src | (uintptr_t)a[0].out) & 15) return false;
    // the positions a tile computes beyond the image rows it owns are wasted MFMA work: take the layer only if at
    // least two thirds of it is useful, and only if the tiles fill a good part of the chip (NSK_HALO_WIDE_ALWAYS:
    // test hook, small shapes)
    if (hooks().halo_wide_always) return true;
    const long long useful = (long long)a[0].Hs * a[0].Ws, computed = (long long)p.tiles_per_img * kNT * 32;
    if (useful * 3 < computed * 2) return false;
    return (long long)a[0].Nimg * p.tiles_per_img * (a[0].Ngemm / block_channels(a[0])) >= 128;
}

int launch_classes(const IgemmArgs *g, int count, hipStream_t stream)
{
    Plan p;
    if (!make_plan(g[0], &p)) return NSK_ERR_BAD_DESC;
    // longest reduction first: the staging of the later channel groups hides behind the first class
    int order[W_CLS];
    for (int i = 0; i < count; ++i) order[i] = i;
    for (int i = 1; i < count; ++i)
        for (int j = i; j > 0 && g[order[j]].ntaps > g[order[j - 1]].ntaps; --j) {
            const int t = order[j];
            order[j] = order[j - 1];
            order[j - 1] = t;
        }
    WideArgs a{};
    const IgemmArgs &f = g[0];
    a.src = f.src; a.out = f.out;
    a.ncls = count;
    for (int i = 0; i < count; ++i) {
        const IgemmArgs &c = g[order[i]];
        a.wpk[i] = c.wpk; a.wpk_bytes[i] = c.wpk_bytes; a.ntaps[i] = c.ntaps;
        a.Mi[i] = c.Mi; a.Mj[i] = c.Mj; a.oa[i] = c.oa; a.ob[i] = c.ob;
        unsigned long long code = 0;
        for (int t = 0; t < c.ntaps; ++t)
            code |= (unsigned long long)((c.add_h + c.off_h[t] + 1) * 4 + (c.add_w + c.off_w[t] + 1)) << (4 * t);
        a.tapcode[i] = code;
    }
    for (int i = count; i < W_CLS; ++i) {
        a.wpk[i] = f.wpk; a.wpk_bytes[i] = 0; a.ntaps[i] = 1;
    }
    a.N = f.Nimg; a.H = f.Hs; a.W = f.Ws; a.C = f.Cs; a.K = f.Ngemm;
    a.Ho = f.Ho; a.Wo = f.Wo; a.Co = f.Co; a.osh = f.osh; a.osw = f.osw;
    a.PW = f.Ws + 2;
    a.rows_per_tile = p.rows_per_tile;
    a.tiles_per_img = p.tiles_per_img;
    a.tiles = f.Nimg * p.tiles_per_img;
    a.n_stage = p.n_stage;
    a.row_bytes = p.row_bytes;
    a.magic_pw = (unsigned)(((1ULL << 32) + a.PW - 1) / a.PW);
    a.src_bytes = f.src_bytes;
    a.out_bytes = (unsigned)((long long)f.Nimg * f.Ho * f.Wo * f.Co * 2);
    a.stats = count == 1 ? f.stats : nullptr;
    a.stats_rows = f.stats_rows;
    static bool attr_set = false;
    if (!attr_set) {
        const void *k[12] = {
            (const void *)conv_halo_wide_kernel<kNT, 4, 0, false>, (const void *)conv_halo_wide_kernel<kNT, 4, 1, false>,
            (const void *)conv_halo_wide_kernel<kNT, 4, 2, false>, (const void *)conv_halo_wide_kernel<kNT, 2, 0, false>,
            (const void *)conv_halo_wide_kernel<kNT, 2, 1, false>, (const void *)conv_halo_wide_kernel<kNT, 2, 2, false>,
            (const void *)conv_halo_wide_kernel<kNT, 4, 0, true>,  (const void *)conv_halo_wide_kernel<kNT, 4, 1, true>,
            (const void *)conv_halo_wide_kernel<kNT, 4, 2, true>,  (const void *)conv_halo_wide_kernel<kNT, 2, 0, true>,
            (const void *)conv_halo_wide_kernel<kNT, 2, 1, true>,  (const void *)conv_halo_wide_kernel<kNT, 2, 2, true>};
        for (int i = 0; i < 12; ++i) {
            const hipError_t e = hipFuncSetAttribute(k[i], hipFuncAttributeMaxDynamicSharedMemorySize, W_LDS_MAX);
            if (e != hipSuccess) {
                set_last_hip_error(e);
                return NSK_ERR_HIP;
            }
        }
        attr_set = true;
    }
    const int bn = block_channels(f);
    const int mode = f.accumulate ? 1 : a.stats ? 2 : 0;
    const bool nine = count == 1 && f.ntaps == 9;
    const dim3 grid((unsigned)(a.tiles * (a.K / bn)));
#define NSK_WIDE_LAUNCH(MW, MODE, NINE) \
    hipLaunchKernelGGL((conv_halo_wide_kernel<kNT, MW, MODE, NINE>), grid, dim3((MW + 1) * 64), p.smem, stream, a)
#define NSK_WIDE_MODES(MW, NINE)                    \
    do {                                            \
        if (mode == 1) NSK_WIDE_LAUNCH(MW, 1, NINE); \
        else if (mode == 2) NSK_WIDE_LAUNCH(MW, 2, NINE); \
        else NSK_WIDE_LAUNCH(MW, 0, NINE);          \
    } while (0)
    if (bn == 128) {
        if (nine) NSK_WIDE_MODES(4, true);
        else NSK_WIDE_MODES(4, false);
    } else {
        if (nine) NSK_WIDE_MODES(2, true);
        else NSK_WIDE_MODES(2, false);
    }
#undef NSK_WIDE_MODES
#undef NSK_WIDE_LAUNCH
    return check_launch();
}

}  // namespace

// One class with all nine taps on its own grid: the forward pass, or the backward-data pass of a stride-1 layer.
bool halo_wide_applicable(int dtype, const IgemmArgs &a)
{
    if (dtype != NSK_BF16 || hooks().no_halo_wide) return false;
    if (a.ntaps != 9 || a.osh != 1 || a.osw != 1 || a.oa != 0 || a.ob != 0) return false;
    if (a.Hs != a.Ho || a.Ws != a.Wo || a.Mi != a.Ho || a.Mj != a.Wo) return false;
    return classes_ok(&a, 1);
}

int halo_wide_stats_rows(const IgemmArgs &a)
{
    Plan p;
    if (a.accumulate || !make_plan(a, &p)) return 0;
    return a.Nimg * p.tiles_per_img;
}

int launch_halo_wide(const IgemmArgs &g, hipStream_t stream) { return launch_classes(&g, 1, stream); }

// The residue classes of a strided backward-data pass (2..4 argument sets on the same tensors), each a stride-1
// convolution over the same source grid with at most nine taps.
bool halo_wide_multi_applicable(int dtype, const IgemmArgs *a, int count)
{
    if (dtype != NSK_BF16 || hooks().no_halo_wide || count < 2) return false;
    for (int i = 0; i < count; ++i)
        if (a[i].stats || a[i].zero_cell) return false;
    return classes_ok(a, count);
}

int launch_halo_wide_multi(const IgemmArgs *a, int count, hipStream_t stream) { return launch_classes(a, count, stream); }

// ---- the forward pass of a 3x3 stride-2 pad-1 layer on even extents: four parity planes of x, staged one after the
// other on the output's own grid, merged into one set of accumulators (MERGE instances of the kernel)
namespace {
// the layer as the stride-1 problem the planner knows: the output grid, x's channels
IgemmArgs s2_as_plane_problem(const IgemmArgs &a)
{
    IgemmArgs v = a;
    v.Hs = a.Mi;
    v.Ws = a.Mj;
    return v;
}
}  // namespace

bool halo_wide_fwd_s2_applicable(int dtype, const IgemmArgs &a)
{
    if (dtype != NSK_BF16 || hooks().no_halo_wide || a.groups > 1 || a.accumulate || a.zero_cell || a.act) return false;
    if (a.ntaps != 9 || (a.Cs != 128 && a.Cs != 256) || a.Ktot != 9 * a.Cs || a.Ngemm % 64 != 0 || a.Co % 8 != 0 || a.Co != a.Ngemm) return false;
    if (a.mult_h != 2 || a.mult_w != 2 || a.add_h != -1 || a.add_w != -1 || a.osh != 1 || a.osw != 1 || a.oa != 0 || a.ob != 0) return false;
    if (a.Hs % 2 != 0 || a.Ws % 2 != 0 || a.Mi != a.Hs / 2 || a.Mj != a.Ws / 2 || a.Ho != a.Mi || a.Wo != a.Mj || a.stats_rows < 0) return false;
    for (int t = 0; t < 9; ++t)
        if (a.off_h[t] != t / 3 || a.off_w[t] != t % 3) return false;
    if ((unsigned long long)a.wpk_bytes >= W_OOB || (((uintptr_t)a.wpk | (uintptr_t)a.src | (uintptr_t)a.out) & 15)) return false;
    const IgemmArgs v = s2_as_plane_problem(a);
    Plan p;
    if (!make_plan(v, &p) || p.n_stage > 288) return false;   // (two moving wavefronts of 144 rows each)
    const long long out_bytes = (long long)a.Nimg * a.Ho * a.Wo * a.Co * 2;
    if ((unsigned long long)a.src_bytes >= W_OOB || out_bytes >= (long long)W_OOB) return false;
    if (hooks().halo_wide_always) return true;
    const long long useful = (long long)v.Hs * v.Ws, computed = (long long)p.tiles_per_img * kNT * 32;
    if (useful * 3 < computed * 2) return false;
    return (long long)a.Nimg * p.tiles_per_img * (a.Ngemm / block_channels(a)) >= 128;
}

int halo_wide_fwd_s2_stats_rows(const IgemmArgs &a)
{
    Plan p;
    if (!make_plan(s2_as_plane_problem(a), &p)) return 0;
    return a.Nimg * p.tiles_per_img;
}

int launch_halo_wide_fwd_s2(const IgemmArgs &g, hipStream_t stream)
{
    const IgemmArgs v = s2_as_plane_problem(g);
    Plan p;
    if (!make_plan(v, &p) || p.n_stage > 288) return NSK_ERR_BAD_DESC;
    WideArgs a{};
    a.src = g.src; a.out = g.out;
    a.ncls = 4;
    // planes in the order of their tap counts (the longest first: the later stages are staged behind it); tap (r, s) of
    // the filter lies on plane (r == 1, s == 1) with shift (r == 2, s == 2)
    static const int plane_a[4] = {0, 0, 1, 1}, plane_b[4] = {0, 1, 0, 1};
    for (int c = 0; c < 4; ++c) {
        a.wpk[c] = g.wpk; a.wpk_bytes[c] = g.wpk_bytes;
        a.Mi[c] = g.Mi; a.Mj[c] = g.Mj; a.oa[c] = 0; a.ob[c] = 0;
        a.pa[c] = plane_a[c]; a.pb[c] = plane_b[c];
        int n = 0;
        unsigned long long code = 0, idx = 0;
        for (int t = 0; t < 9; ++t) {
            const int r = t / 3, sc = t % 3;
            if ((r == 1) != (plane_a[c] == 1) || (sc == 1) != (plane_b[c] == 1)) continue;
            const int dh = r == 2 ? 1 : 0, dw = sc == 2 ? 1 : 0;
            code |= (unsigned long long)((dh + 1) * 4 + (dw + 1)) << (4 * n);
            idx |= (unsigned long long)t << (4 * n);
            ++n;
        }
        a.ntaps[c] = n; a.tapcode[c] = code; a.tapidx[c] = idx;
    }
    a.wrow_taps = 9;
    a.Hx = g.Hs; a.Wx = g.Ws;
    a.N = g.Nimg; a.H = v.Hs; a.W = v.Ws; a.C = g.Cs; a.K = g.Ngemm;
    a.Ho = g.Ho; a.Wo = g.Wo; a.Co = g.Co; a.osh = 1; a.osw = 1;
    a.PW = v.Ws + 2;
    a.rows_per_tile = p.rows_per_tile;
    a.tiles_per_img = p.tiles_per_img;
    a.tiles = g.Nimg * p.tiles_per_img;
    a.n_stage = p.n_stage;
    a.row_bytes = p.row_bytes;
    a.magic_pw = (unsigned)(((1ULL << 32) + a.PW - 1) / a.PW);
    a.src_bytes = g.src_bytes;
    a.out_bytes = (unsigned)((long long)g.Nimg * g.Ho * g.Wo * g.Co * 2);
    a.stats = g.stats;
    a.stats_rows = g.stats_rows;
    if (g.stats && g.stats_rows != a.tiles) return NSK_ERR_BAD_DESC;   // the planner and the launch disagree
    static bool attr_set = false;
    if (!attr_set) {
        const void *k[4] = {
            (const void *)conv_halo_wide_kernel<kNT, 4, 0, false, true>, (const void *)conv_halo_wide_kernel<kNT, 4, 2, false, true>,
            (const void *)conv_halo_wide_kernel<kNT, 2, 0, false, true>, (const void *)conv_halo_wide_kernel<kNT, 2, 2, false, true>};
        for (int i = 0; i < 4; ++i) {
            const hipError_t e = hipFuncSetAttribute(k[i], hipFuncAttributeMaxDynamicSharedMemorySize, W_LDS_MAX);
            if (e != hipSuccess) {
                set_last_hip_error(e);
                return NSK_ERR_HIP;
            }
        }
        attr_set = true;
    }
    const int bn = block_channels(g);
    const dim3 grid((unsigned)(a.tiles * (a.K / bn)));
    if (bn == 128) {
        if (a.stats)
            hipLaunchKernelGGL((conv_halo_wide_kernel<kNT, 4, 2, false, true>), grid, dim3(6 * 64), p.smem, stream, a);
        else
            hipLaunchKernelGGL((conv_halo_wide_kernel<kNT, 4, 0, false, true>), grid, dim3(6 * 64), p.smem, stream, a);
    } else {
        if (a.stats)
            hipLaunchKernelGGL((conv_halo_wide_kernel<kNT, 2, 2, false, true>), grid, dim3(4 * 64), p.smem, stream, a);
        else
            hipLaunchKernelGGL((conv_halo_wide_kernel<kNT, 2, 0, false, true>), grid, dim3(4 * 64), p.smem, stream, a);
    }
    return check_launch();
}

}  // namespace nsk

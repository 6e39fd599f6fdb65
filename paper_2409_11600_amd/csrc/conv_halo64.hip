// 3x3, stride 1, 64 -> 64 channel bf16 convolution (forward, and backward-data through the packed
// transposed filter): the layer shape that carries most of the 3x3 FLOPs of the residual networks the
// paper trains (section "Experiments and Discussion").
//
// Why a second kernel.  On gfx950 a bf16 32x32x16 MFMA lasts 32 clocks, so an instruction stream may
// spend only a handful of other vector instructions per MFMA, and a k-tile that is re-staged from
// L2 for each of the nine taps saturates the L1 fill bandwidth of a CU.  This kernel therefore
//   * keeps the whole packed filter (64 x 9 x 64 bf16 = 72 KB) resident in LDS for the life of the
//     block (the 160 KB LDS of a CU makes that possible),
//   * stages each input tile ONCE, with its halo, and reads the nine taps as shifted LDS rows,
//   * is persistent: a block walks over many tiles, prefetching the next tile into registers while
//     the MFMAs of the current one run, so no per-block prologue is paid per tile.
//
// Flat padded coordinates.  Every image is viewed as a zero-padded (H+2) x (W+2) grid and all images
// are laid end to end; position q = img*(H+2)*(W+2) + hp*(W+2) + wp.  A tap (dh, dw) is then the same
// constant shift dh*(W+2) + dw for every position, image borders need no special case (padding
// positions load zeros through an out-of-range buffer offset), and a tile is simply 256 consecutive
// positions.  Outputs computed at padding positions are discarded; that wastes
// ((H+2)(W+2) - HW)/HW of the MFMA work (7% at 56 x 56).
//
// Block = 256 threads = 4 wavefronts, each owning 64 positions x 64 output channels as 2 x 2
// accumulators of 32x32.  LDS rows are padded (144 B per position, 1168 B per filter row) so that the
// 16-byte fragment reads of 8 consecutive rows cover all banks once.
#include <stdlib.h>

#include "nsk_internal.h"

namespace nsk {
namespace {

constexpr int HT = 256;            // positions per tile
constexpr int H_MAX_IN = 400;      // staged positions incl. halo: HT + 2*(W+3) <= 400  ->  W <= 69
constexpr int H_IN_STRIDE = 144;   // bytes per staged position (64 ch bf16 + 16 pad)
constexpr int H_W_STRIDE = 1168;   // bytes per filter row (9*64 bf16 + 16 pad)
constexpr int H_PASSES = (H_MAX_IN + 31) / 32;
constexpr unsigned H_OOB = 0xF0000000u;

struct HaloArgs {
    const void *src, *wpk;
    void *out;
    int N, H, W;
    int PW, PI;               // padded width, padded image size
    int total_pos, tiles, halo;
    unsigned long long magic_pi, magic_pw;  // ceil(2^40 / d)
    unsigned src_bytes, out_bytes;
    int accumulate;
    int tapoff[9];            // shift of each tap in flat padded positions
    float *stats;             // two-group kernel only: per-channel partial sums of the stored output, or nullptr
    int stats_rows;           // 8 rows per block (one per wavefront)
};

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

template <bool ACCUM>
__global__ __launch_bounds__(256) void conv_halo64_kernel(const HaloArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char *in_lds = smem;                                    // H_MAX_IN * 144
    unsigned char *w_lds = smem + H_MAX_IN * H_IN_STRIDE;            // 64 * 1168
    unsigned *out_tab = (unsigned *)(w_lds + 64 * H_W_STRIDE);       // 256 byte offsets
    unsigned *in_tab = out_tab + 256;                                // H_MAX_IN byte offsets
    unsigned char *st_lds = (unsigned char *)(in_tab + H_MAX_IN);    // 4 wavefronts x 32 positions x 144 B

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int frow = lane & 31, fk = lane >> 5;
    const __amdgpu_buffer_rsrc_t src_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.src, 0, a.src_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t out_rsrc = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, a.out_bytes, 0x00020000);

    // filter -> LDS, once per block: 64 rows x 72 vectors
    {
        const u32x4 *w = (const u32x4 *)a.wpk;
        u32x4 tmp[18];   // 64 * 72 / 256 vectors per thread, all loads in flight before the first write
#pragma unroll
        for (int u = 0; u < 18; ++u) tmp[u] = w[tid + 256 * u];
#pragma unroll
        for (int u = 0; u < 18; ++u) {
            const int i = tid + 256 * u, row = i / 72, v = i - row * 72;
            *(u32x4 *)(w_lds + row * H_W_STRIDE + v * 16) = tmp[u];
        }
    }

    const int n_in = HT + 2 * a.halo;        // staged positions of a tile
    const int chunk = tid & 7, prow = tid >> 3;

    // byte offset of padded position q (channel chunk `chunk`) in the NHWC tensor, or out of range
    auto src_offset = [&](int q) -> unsigned {
        // branch-free: an invalid position is clamped for the arithmetic and replaced at the end
        const bool inside = (unsigned)q < (unsigned)a.total_pos;
        const unsigned qq = inside ? (unsigned)q : 0u;
        const unsigned img = (unsigned)(((unsigned long long)qq * a.magic_pi) >> 40);
        const unsigned rem = qq - img * (unsigned)a.PI;
        const unsigned hp = (unsigned)(((unsigned long long)rem * a.magic_pw) >> 40);
        const unsigned wp = rem - hp * (unsigned)a.PW;
        const bool ok = inside & (hp - 1u < (unsigned)a.H) & (wp - 1u < (unsigned)a.W);
        const unsigned off = (((img * a.H + (hp - 1u)) * a.W + (wp - 1u)) * 64u) * 2u;
        return ok ? off : H_OOB;
    };

    // Two register sets: while tile t is multiplied, tile t+G is already in (or on its way into) one
    // set and the loads of tile t+2G are issued into the set that tile t has just vacated.  HBM latency
    // under load (several microseconds) is longer than the matrix work of one tile.
    u32x4 stageA[H_PASSES], stageB[H_PASSES];
    // one of the H_PASSES 16-byte loads of a tile's staged input (8 lanes per position)
    // in_tab[p] = byte offset of staged position p of the tile being prefetched (or out of range):
    // computed by two positions per thread, so the eight lanes that share a position do not repeat
    // the index arithmetic and a prefetch step is one table read, one add and one load.
    auto fill_in_tab = [&](int tile) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int p = tid + 256 * u;
            if (p < H_MAX_IN) in_tab[p] = p < n_in ? src_offset(tile * HT - a.halo + p) : H_OOB;
        }
    };
    // The table is read in one batch (LDS returns in order, so a table read in the middle of the MFMA
    // loop would force a wait on the fragment reads issued before it); a prefetch step is then one load.
    unsigned poff[H_PASSES];
    auto read_in_tab = [&]() {
#pragma unroll
        for (int u = 0; u < H_PASSES; ++u) {
            const unsigned off = in_tab[u * 32 + prow];
            poff[u] = off == H_OOB ? H_OOB : off + chunk * 16;
        }
    };
    auto prefetch_piece = [&](u32x4 (&S)[H_PASSES], int u) { S[u] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, poff[u], 0, 0); };

    // each block owns a contiguous run of tiles: the halo a tile shares with its successor was fetched by
    // this same CU moments ago and is still in its L2 (a strided assignment re-fetched every halo from HBM)
    constexpr int G = 1;
    const int tiles_per_block = (a.tiles + (int)gridDim.x - 1) / (int)gridDim.x;
    const int t_end = min(a.tiles, ((int)blockIdx.x + 1) * tiles_per_block);
    int tile = blockIdx.x * tiles_per_block;
    if (tile < t_end) {
        fill_in_tab(tile);
        lds_barrier();
        read_in_tab();
#pragma unroll
        for (int u = 0; u < H_PASSES; ++u) prefetch_piece(stageA, u);
        lds_barrier();
        if (tile + G < t_end) {
            fill_in_tab(tile + G);
            lds_barrier();
            read_in_tab();
#pragma unroll
            for (int u = 0; u < H_PASSES; ++u) prefetch_piece(stageB, u);
        }
    }

    const unsigned a_base0 = (unsigned)((wave * 64 + frow + a.halo) * H_IN_STRIDE + fk * 16);
    const unsigned b_base0 = (unsigned)(frow * H_W_STRIDE + fk * 16);
    unsigned char *my_st = st_lds + wave * (32 * H_IN_STRIDE);

    auto do_tile = [&](int tile, u32x4 (&stage)[H_PASSES]) {
        // staged registers -> LDS (the barrier at the end of the previous tile freed the buffer)
#pragma unroll
        for (int u = 0; u < H_PASSES; ++u) {
            const int p = u * 32 + prow;
            if (p < n_in) *(u32x4 *)(in_lds + p * H_IN_STRIDE + chunk * 16) = stage[u];
        }
        out_tab[tid] = src_offset(tile * HT + tid);   // the output tensor has the same geometry
        const int next = tile + 2 * G;                // the tile whose loads go into the set just emptied
        const bool have_next = next < t_end;
        if (have_next) fill_in_tab(next);   // the previous tile's reads of in_tab are complete
        lds_barrier();
        if (have_next) {
            read_in_tab();
        } else {
#pragma unroll
            for (int u = 0; u < H_PASSES; ++u) poff[u] = H_OOB;
        }

        // The filter rows are the MFMA "A" operand and the positions the "B" operand, so a lane ends up
        // with 4 CONSECUTIVE CHANNELS of one position per accumulator quad: acc[ni][mi][4g+j] is channel
        // 32*ni + 8*g + 4*(lane/32) + j of position 32*mi + lane%32.
        f32x16 acc[2][2];
        if (ACCUM) {
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) {
                const unsigned off = out_tab[wave * 64 + mi * 32 + frow];
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const unsigned o = off == H_OOB ? H_OOB : off + (unsigned)((ni * 32 + g * 8 + fk * 4) * 2);
                        const u32x2 old = __builtin_amdgcn_raw_buffer_load_b64(out_rsrc, o, 0, 0);
                        const bf16x4 ob = __builtin_bit_cast(bf16x4, old);
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj) acc[ni][mi][g * 4 + jj] = (float)ob[jj];
                    }
            }
        } else {
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[ni][mi][v] = 0.f;
        }

        // 36 reduction steps (9 taps x 4 groups of 16 channels).  One wavefront per SIMD means nobody
        // else hides LDS latency, so fragments are fetched two steps ahead into a rotating set of
        // registers; the scheduling barriers keep the compiler from sinking the reads back to their use.
        // The loads of the NEXT tile are issued one per step, in the shadow of the MFMAs.
        unsigned ta[9];
#pragma unroll
        for (int t = 0; t < 9; ++t) ta[t] = a_base0 + (unsigned)(a.tapoff[t] * H_IN_STRIDE);
        bf16x8 af[3][2], bfr[3][2];
        auto fetch = [&](int step, int set) {
            const int t = step >> 2, kc = step & 3;
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
                af[set][mi] = *(const bf16x8 *)(in_lds + ta[t] + mi * 32 * H_IN_STRIDE + kc * 32);
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
                bfr[set][ni] = *(const bf16x8 *)(w_lds + b_base0 + ni * 32 * H_W_STRIDE + (t * 64 + kc * 16) * 2);
        };
        fetch(0, 0);
        fetch(1, 1);
#pragma unroll
        for (int step = 0; step < 36; ++step) {
            if (step + 2 < 36) fetch(step + 2, (step + 2) % 3);
            if (step < H_PASSES) prefetch_piece(stage, step);   // unconditional: without a next tile the offsets are out of range
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
                    acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[step % 3][ni], af[step % 3][mi], acc[ni][mi], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }

        // Epilogue: round to bf16, transpose through this wavefront's private LDS strip so that every
        // lane stores 16 contiguous bytes (8 lanes cover the 128 bytes of one position).
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x4 pk;
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) pk[jj] = (bf16_t)acc[ni][mi][g * 4 + jj];
                    *(bf16x4 *)(my_st + frow * H_IN_STRIDE + (ni * 32 + g * 8 + fk * 4) * 2) = pk;
                }
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const int idx = lane + 64 * jj, pos = idx >> 3, ck = idx & 7;
                const u32x4 v = *(const u32x4 *)(my_st + pos * H_IN_STRIDE + ck * 16);
                const unsigned off = out_tab[wave * 64 + mi * 32 + pos];
                const unsigned o = off == H_OOB ? H_OOB : off + (unsigned)(ck * 16);
                __builtin_amdgcn_raw_buffer_store_b128(v, out_rsrc, o, 0, 0);
            }
        }
        lds_barrier();
    };
    for (; tile < t_end; tile += 2 * G) {
        do_tile(tile, stageA);
        if (tile + G < t_end) do_tile(tile + G, stageB);
    }
}


// ---------------------------------------------------------------------------------------------------
// Two-group ("ping-pong") variant.  In the kernel above the four wavefronts stage, multiply and store
// one after the other, so the matrix units idle during staging and the epilogue (about 45% of a tile's
// time).  Here a block has EIGHT wavefronts in two groups of four that share the resident filter.  In
// phase p one group multiplies tile p while the other stores tile p-1 and stages the input rows tile p+1
// will need; one block-wide barrier per phase, and the groups swap roles.  Two wavefronts share each SIMD,
// so the vector, LDS and memory instructions of one run in the shadow of the other's MFMAs.
//
// Input ring.  Consecutive tiles of a block overlap by their halos, so the staged positions live in a
// ring of RING = 512 + 2*halo slots of 128 bytes: tile p reads ring rows [256p, 256p + 256 + 2*halo), and
// the 256 rows staged in phase p (for tile p+1) land exactly on the rows tile p-1 has just finished with.
// Those same dead rows, split into four private 64-slot strips, first serve as the transposing buffer of
// the storing group's epilogue, so no wavefront ever needs another's LDS data inside a phase.
// Slots are not padded; the 16-byte chunk index is XOR-ed with bits 1..3 of the slot number, which makes
// the fragment reads of 16 consecutive slots hit all 64 banks once.
constexpr int P_RING_MAX = 640;    // 512 + 2*halo <= 640  ->  W <= 61
constexpr int P_SLOT = 128;

template <bool ACCUM>
__global__ __launch_bounds__(512) void conv_halo64_pp_kernel(const HaloArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char *ring = smem;                                  // P_RING_MAX * 128
    unsigned char *w_lds = smem + P_RING_MAX * P_SLOT;           // 64 * 1168

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave >> 2, x = wave & 3;
    const int frow = lane & 31, fk = lane >> 5;
    const int prow = lane >> 3, chunk = lane & 7;
    const __amdgpu_buffer_rsrc_t src_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.src, 0, a.src_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t out_rsrc = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, a.out_bytes, 0x00020000);

    const int tiles_per_block = (a.tiles + (int)gridDim.x - 1) / (int)gridDim.x;
    const int T0 = blockIdx.x * tiles_per_block;
    const int n = min(a.tiles, T0 + tiles_per_block) - T0;      // tiles of this block
    // Statistics epilogue (forward only): every lane adds up the 8 channels of its 16-byte pieces over all the
    // positions it stores during the life of the block; one cross-lane reduction and one row per wavefront at the end.
    float ssum[8], ssq[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) ssum[e] = ssq[e] = 0.f;
    auto write_stats = [&]() {
        if (!a.stats) return;
#pragma unroll
        for (int e = 0; e < 8; ++e)
#pragma unroll
            for (int o = 8; o < 64; o <<= 1) {
                ssum[e] += __shfl_xor(ssum[e], o, 64);
                ssq[e] += __shfl_xor(ssq[e], o, 64);
            }
        if (lane < 8) {
            float *r0 = a.stats + (size_t)(blockIdx.x * 8 + wave) * 64 + lane * 8;
            float *r1 = r0 + (size_t)a.stats_rows * 64;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                r0[e] = ssum[e];
                r1[e] = ssq[e];
            }
        }
    };
    if (n <= 0) {                                                // uniform for the block: no barrier is skipped
        write_stats();                                           // zeros: every row of the buffer is written
        return;
    }
    const unsigned RING = 512u + 2u * (unsigned)a.halo;
    const int Q0 = T0 * HT - a.halo;                             // padded position held by ring row 0

    auto src_offset = [&](int q) -> unsigned {
        const bool inside = (unsigned)q < (unsigned)a.total_pos;
        const unsigned qq = inside ? (unsigned)q : 0u;
        const unsigned img = (unsigned)(((unsigned long long)qq * a.magic_pi) >> 40);
        const unsigned rem = qq - img * (unsigned)a.PI;
        const unsigned hp = (unsigned)(((unsigned long long)rem * a.magic_pw) >> 40);
        const unsigned wp = rem - hp * (unsigned)a.PW;
        const bool ok = inside & (hp - 1u < (unsigned)a.H) & (wp - 1u < (unsigned)a.W);
        const unsigned off = (((img * a.H + (hp - 1u)) * a.W + (wp - 1u)) * 64u) * 2u;
        return ok ? off : H_OOB;
    };
    // s < 2*RING  ->  s mod RING  (s - RING wraps to a huge value when s < RING)
    auto wrap = [&](unsigned s) -> unsigned { return min(s, s - RING); };
    auto slot_addr = [&](unsigned slot, unsigned c) -> unsigned { return slot * P_SLOT + ((c ^ ((slot >> 1) & 7u)) << 4); };
    // Byte offsets of 64 consecutive padded positions starting at q_first, as this lane needs them for
    // its eight 16-byte pieces (piece u = position prow + 8u, channel chunk `chunk`): lane L does the index
    // arithmetic for position L and the results are exchanged across lanes.  An out-of-range marker stays
    // out of range after the chunk offset is added.
    auto row_offsets = [&](int q_first, bool valid, unsigned (&off)[8]) {
        const unsigned mine = valid ? src_offset(q_first + lane) : H_OOB;
#pragma unroll
        for (int u = 0; u < 8; ++u)
            off[u] = (unsigned)__builtin_amdgcn_ds_bpermute((prow + 8 * u) * 4, (int)mine) + (unsigned)(chunk * 16);
    };

    // prologue: the filter (64 rows x 72 vectors) and ring rows [0, 384), which cover everything tile 0
    // needs (256 + 2*halo <= 384 rows); all loads are in flight before the first LDS write
    {
        unsigned off[8];
        row_offsets(Q0 + 64 * wave, wave < 6, off);
        u32x4 v[8], tmp[9];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, off[u], 0, 0);
        const u32x4 *w = (const u32x4 *)a.wpk;
#pragma unroll
        for (int u = 0; u < 9; ++u) tmp[u] = w[tid + 512 * u];
        if (wave < 6) {
#pragma unroll
            for (int u = 0; u < 8; ++u)
                *(u32x4 *)(ring + slot_addr((unsigned)(64 * wave + prow + 8 * u), (unsigned)chunk)) = v[u];
        }
#pragma unroll
        for (int u = 0; u < 9; ++u) {
            const int i = tid + 512 * u, row = i / 72, vv = i - row * 72;
            *(u32x4 *)(w_lds + row * H_W_STRIDE + vv * 16) = tmp[u];
        }
    }

    // Staging unit u = ring rows [2*halo + 256(u-1), 2*halo + 256u): the rows tile u-1 needs beyond those
    // of tile u-2.  A wavefront stages 64 of them; units past the block's last tile load nothing.
    u32x4 st[8];
    auto issue = [&](int unit) {
        unsigned off[8];
        row_offsets(Q0 + 2 * a.halo + 256 * (unit - 1) + 64 * x, unit <= n, off);
#pragma unroll
        for (int u = 0; u < 8; ++u) st[u] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, off[u], 0, 0);
    };
    unsigned ss = grp ? (unsigned)(2 * a.halo + 256 + 64 * x) : (unsigned)(64 * x);   // first slot of this wavefront's strip
    unsigned cs = (unsigned)(256 * grp);                                              // ring slot of row 0 of the next tile to multiply
    issue(grp ? 2 : 3);

    const unsigned b_base0 = (unsigned)(frow * H_W_STRIDE + fk * 16);
    f32x16 acc[2][2];
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // LDS address of this lane's input fragment for tap t, position tile mi, channel group 0 of the next
    // tile this group multiplies; prepared outside the multiply phase, which then only XORs in the group
    unsigned ta[9][2];
    auto prepare_ta = [&]() {
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) {
                const unsigned r = wrap(cs + (unsigned)(x * 64 + mi * 32 + frow + a.halo + a.tapoff[t]));
                ta[t][mi] = r * P_SLOT + (((unsigned)fk ^ ((r >> 1) & 7u)) << 4);
            }
    };
    prepare_ta();
    lds_barrier();

    for (int p = 0; p <= n; ++p) {
        if ((p & 1) == grp) {
            if (p < n) {
                // ---- multiply tile p: 36 reduction steps (9 taps x 4 groups of 16 channels), fragments
                // fetched two steps ahead into a rotating register set
                bf16x8 af[3][2], bfr[3][2];
                auto fetch = [&](int step, int set) {
                    const int t = step >> 2, kc = step & 3;
#pragma unroll
                    for (int mi = 0; mi < 2; ++mi) af[set][mi] = *(const bf16x8 *)(ring + (ta[t][mi] ^ (unsigned)(kc << 5)));
#pragma unroll
                    for (int ni = 0; ni < 2; ++ni)
                        bfr[set][ni] = *(const bf16x8 *)(w_lds + b_base0 + ni * 32 * H_W_STRIDE + (t * 64 + kc * 16) * 2);
                };
                // the multiplying wavefront goes first whenever both wavefronts of a SIMD are ready
                __builtin_amdgcn_s_setprio(3);
                fetch(0, 0);
                fetch(1, 1);
#pragma unroll
                for (int step = 0; step < 36; ++step) {
                    if (step + 2 < 36) fetch(step + 2, (step + 2) % 3);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                        for (int ni = 0; ni < 2; ++ni)
                            acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[step % 3][ni], af[step % 3][mi],
                                                                                  step == 0 ? zero16 : acc[ni][mi], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
                __builtin_amdgcn_s_setprio(0);
                cs = wrap(cs + 512u);
            }
        } else {
            if (p >= 1) {
                // ---- store tile p-1.  acc[ni][mi][4g+j] is channel 32ni + 8g + 4fk + j of position 32mi + frow;
                // transposed through the private strip so that a lane stores 16 contiguous bytes.
                unsigned ooff[8];
                row_offsets((T0 + p - 1) * HT + 64 * x, true, ooff);
                if (ACCUM) {
                    // fp32 through the strip (two slots per position), 32 positions at a time, so the sum
                    // with the old value is rounded once
#pragma unroll
                    for (int mi = 0; mi < 2; ++mi) {
                        u32x4 old[4];
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj) old[jj] = __builtin_amdgcn_raw_buffer_load_b128(out_rsrc, ooff[mi * 4 + jj], 0, 0);
#pragma unroll
                        for (int ni = 0; ni < 2; ++ni) {
                            const unsigned sl = wrap(ss + (unsigned)(2 * frow + ni));
#pragma unroll
                            for (int g = 0; g < 4; ++g) {
                                f32x4 v;
#pragma unroll
                                for (int jj = 0; jj < 4; ++jj) v[jj] = acc[ni][mi][g * 4 + jj];
                                *(f32x4 *)(ring + slot_addr(sl, (unsigned)(2 * g + fk))) = v;
                            }
                        }
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj) {
                            const int pos = prow + 8 * jj;     // position within this half; channels 8*chunk..+7
                            const unsigned sl = wrap(ss + (unsigned)(2 * pos + (chunk >> 2)));
                            const f32x4 lo = *(const f32x4 *)(ring + slot_addr(sl, (unsigned)(2 * (chunk & 3))));
                            const f32x4 hi = *(const f32x4 *)(ring + slot_addr(sl, (unsigned)(2 * (chunk & 3) + 1)));
                            const bf16x8 ob = __builtin_bit_cast(bf16x8, old[jj]);
                            bf16x8 r;
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                r[e] = (bf16_t)(lo[e] + (float)ob[e]);
                                r[4 + e] = (bf16_t)(hi[e] + (float)ob[4 + e]);
                            }
                            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, r), out_rsrc, ooff[mi * 4 + jj], 0, 0);
                        }
                    }
                } else {
#pragma unroll
                    for (int mi = 0; mi < 2; ++mi) {
                        const unsigned sl = wrap(ss + (unsigned)(mi * 32 + frow));
#pragma unroll
                        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                            for (int g = 0; g < 4; ++g) {
                                bf16x4 pk;
#pragma unroll
                                for (int jj = 0; jj < 4; ++jj) pk[jj] = (bf16_t)acc[ni][mi][g * 4 + jj];
                                *(bf16x4 *)(ring + slot_addr(sl, (unsigned)(ni * 4 + g)) + fk * 8) = pk;
                            }
                    }
#pragma unroll
                    for (int jj = 0; jj < 8; ++jj) {
                        const unsigned sl = wrap(ss + (unsigned)(prow + 8 * jj));
                        const u32x4 v = *(const u32x4 *)(ring + slot_addr(sl, (unsigned)chunk));
                        __builtin_amdgcn_raw_buffer_store_b128(v, out_rsrc, ooff[jj], 0, 0);
                        if (a.stats) {
                            const float live = ooff[jj] < H_OOB ? 1.f : 0.f;   // padding positions are not stored
                            const bf16x8 vb = __builtin_bit_cast(bf16x8, v);
#pragma unroll
                            for (int e = 0; e < 8; ++e) {
                                const float f = live * (float)vb[e];
                                ssum[e] += f;
                                ssq[e] += f * f;
                            }
                        }
                    }
                }
            }
            if (p + 1 < n) {
                // ---- commit the rows loaded two phases ago (tile p+1 reads them in the next phase)
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    *(u32x4 *)(ring + slot_addr(wrap(ss + (unsigned)(prow + 8 * u)), (unsigned)chunk)) = st[u];
            }
            ss = wrap(ss + 512u);
            issue(p + 4);
            prepare_ta();
        }
        lds_barrier();
    }
    write_stats();
}


// ---------------------------------------------------------------------------------------------------
// Filter-stationary variant.  In the two kernels above every multiply step reads its two filter
// fragments AND its two input fragments from LDS: four 1 KB reads per four MFMAs and wavefront, which is
// the whole LDS bandwidth of a CU (128 bytes per clock) when four wavefronts multiply, so the matrix
// units wait for LDS about half of the time.  Here a block has FOUR wavefronts, one per SIMD, each with
// the 512-register budget of a lone wavefront, and every wavefront keeps the WHOLE packed filter in
// registers for the life of the block (36 reduction steps x 2 halves of the output channels x 4
// registers = 288; 256 of them in the accumulation-register half of the file, which the MFMAs read
// directly, the accumulators themselves in ordinary registers).  Only the input fragments come from
// LDS: one 1 KB read per two MFMAs, half of the LDS bandwidth, and the filter does not occupy LDS.
//
// A wavefront owns MI x 32 positions x 64 output channels of each tile (tile = 128*MI positions).  With
// one wavefront per SIMD nothing else can fill the matrix pipe while a wavefront does something else, and
// a wavefront issues in order: whatever stands between two MFMAs and takes longer than the 32 clocks of
// the first one idles the matrix unit.  So the work around the MFMAs is cut into pieces of a few
// instructions that sit between the MFMAs of the multiply loop (fully unrolled, 36 steps): after its last
// MFMA a wavefront only converts its accumulators to bf16 and drops them into a private LDS strip
// (position-major, the transposition for 16-byte stores); reading the strip back, the output offsets, the
// global stores and the statistics sums happen inside the multiply loop of the NEXT tile, as do the index
// arithmetic and the global loads of the input rows the tile after that needs, and their LDS writes.
// One LDS-only barrier per tile.
//
// Input ring: as above, RING = 2*tile + 2*halo rows (rows of 144 bytes: padded instead of swizzled, so a
// fragment address is slot*144 + constant and the channel-group offset is an immediate).  Tile p reads ring
// rows [tile*p, tile*p + tile + 2*halo); the rows written during tile p (for tile p+1) land on rows that
// only tile p-1 used.
//
// Start of a block: the filter is fetched ONCE per block (256 threads, 18 coalesced 16-byte loads each),
// passed through LDS (the ring's space, rows padded to 1168 bytes) and read back by every wavefront in
// operand layout; the input rows of the first tile are requested before that and written to the ring after.
constexpr int F_SLOT = 144;
constexpr int F_RING_MAX = 512 + 128;   // rows: 2*256 + 2*halo, halo <= 64
constexpr int F_AGPR_STEPS = 24;        // reduction steps whose filter fragments live in accumulation registers (8 each; the accumulators take the other 64)

// The multiply work of a tile of the filter-stationary kernel is a sequence of 36*MI "pairs": pair = (reduction step,
// position tile mi), two MFMAs (the two halves of the output channels) on one input fragment.  With two position tiles
// the first two and the last two taps run position tile 0 first (eight steps, sixteen MFMAs) and then position tile 1,
// so that the accumulators of a position tile are complete, or not yet needed, while sixteen MFMAs of the other one
// run: that is where the conversion of the accumulators to bf16 and their LDS writes go.
template <int MI> constexpr int fs_pair_step(int pair)
{
    if (MI == 1) return pair;
    if (pair < 16) return pair & 7;
    if (pair >= 56) return 28 + (pair & 7);
    return 8 + ((pair - 16) >> 1);
}
template <int MI> constexpr int fs_pair_mi(int pair)
{
    if (MI == 1) return 0;
    if (pair < 16) return pair >> 3;
    if (pair >= 56) return (pair - 56) >> 3;
    return pair & 1;
}

// The side work of a tile as a list of small actions.  The slot in front of the first MFMA of a pair holds the read of an
// input fragment four pairs ahead (and, with statistics, a few additions); the slot in front of the second MFMA of pair m
// holds action m of this list (and the steps of the output pipeline below):
//   TAP        LDS address of a later tap's fragments for one position tile, before the first read that needs it
//   FA.. FB3   byte offsets of the previous tile's outputs: index arithmetic in five pieces
//   IA.. IBP   byte offsets of the input rows of the tile after the next: the same, and the lane exchange
//   CL         one 16-byte piece of the input rows requested during the previous tile goes to the ring (a row of the
//              next tile), and the same registers are requested again for the tile after that: a request has a
//              whole tile's time (2.5 us) to come back from HBM
enum { F_NONE, F_TAP, F_IA1, F_IA2, F_IB1, F_IB2, F_IB3, F_IBP, F_FA1, F_FA2, F_FB1, F_FB2, F_FB3, F_CL };
struct FsAct { int kind, arg; };   // arg of TAP: 2*tap + mi
template <int MI> constexpr FsAct fs_action(int m)
{
    if (MI == 2) {
        switch (m) {
        case 0: return {F_TAP, 2 * 1 + 1};
        case 8: return {F_TAP, 2 * 2}; case 9: return {F_TAP, 2 * 2 + 1}; case 16: return {F_TAP, 2 * 3}; case 17: return {F_TAP, 2 * 3 + 1};
        case 24: return {F_TAP, 2 * 4}; case 25: return {F_TAP, 2 * 4 + 1}; case 32: return {F_TAP, 2 * 5}; case 33: return {F_TAP, 2 * 5 + 1};
        case 40: return {F_TAP, 2 * 6}; case 41: return {F_TAP, 2 * 6 + 1}; case 48: return {F_TAP, 2 * 7}; case 49: return {F_TAP, 2 * 7 + 1};
        case 51: return {F_TAP, 2 * 8}; case 52: return {F_TAP, 2 * 8 + 1};
        case 1: return {F_FA1, 0}; case 2: return {F_FA2, 0}; case 3: return {F_FB1, 0}; case 4: return {F_FB2, 0}; case 5: return {F_FB3, 0};
        case 6: return {F_IA1, 0}; case 7: return {F_IA2, 0}; case 10: return {F_IB1, 0}; case 11: return {F_IB2, 0}; case 12: return {F_IB3, 0};
        case 13: return {F_IBP, 0}; case 14: return {F_IBP, 1};
        case 18: return {F_CL, 0}; case 20: return {F_CL, 1}; case 21: return {F_CL, 2}; case 22: return {F_CL, 3};
        case 26: return {F_CL, 4}; case 28: return {F_CL, 5}; case 29: return {F_CL, 6}; case 30: return {F_CL, 7};
        default: return {F_NONE, 0};
        }
    }
    if (m < 28 && m % 4 == 1) return {F_TAP, ((m + 7) / 4) * 2};                // tap (m + 7)/4 = 2 .. 8
    switch (m) {
    case 0: return {F_FA1, 0}; case 2: return {F_FA2, 0}; case 3: return {F_FB1, 0}; case 4: return {F_FB2, 0}; case 6: return {F_FB3, 0};
    case 7: return {F_IA1, 0}; case 8: return {F_IA2, 0}; case 10: return {F_IB1, 0}; case 11: return {F_IB2, 0}; case 12: return {F_IB3, 0};
    case 14: return {F_IBP, 0};
    case 27: return {F_CL, 0}; case 28: return {F_CL, 1}; case 30: return {F_CL, 2}; case 31: return {F_CL, 3};
    default: return {F_NONE, 0};
    }
}
// The outputs of the previous tile leave one 16-byte vector at a time: vector g is read back from the strip (and its byte
// offset fetched from the lane that computed it) in the side slot of pair fs_out_first + S*g, stored two (one) pairs
// later, and, with statistics, added up in the fragment-read slots of the pairs after that (MI = 2: one dword per slot,
// four slots; MI = 1: the four dwords in one slot).
template <int MI> constexpr int fs_out_first() { return 15; }
template <int MI> constexpr int fs_out_every() { return MI == 2 ? 4 : 3; }
template <int MI> constexpr int fs_out_read(int pair)    // vector whose strip read sits in this pair's side slot, or -1
{
    const int d = pair - fs_out_first<MI>();
    return d >= 0 && d % fs_out_every<MI>() == 0 && d / fs_out_every<MI>() < 4 * MI ? d / fs_out_every<MI>() : -1;
}
template <int MI> constexpr int fs_out_store(int pair) { return fs_out_read<MI>(pair - (MI == 2 ? 2 : 1)); }
template <int MI> constexpr int fs_out_count(int pair)   // first dword (4*g + d) counted in this pair's read slot, or -1
{
    if (MI == 2) {
        const int d = pair - (fs_out_first<MI>() + 3);
        return d >= 0 && d < 32 ? d : -1;
    }
    const int g = fs_out_read<MI>(pair - 2);
    return g >= 0 ? 4 * g : -1;
}
// Position tile 1 of the previous tile is converted in front of MFMAs 2, 4, .., 16 (position tile 0 is being multiplied),
// position tile 0 of this tile in front of MFMAs 130, 132, .., 142 and 143 (its last MFMA is number 127).
constexpr int fs_epilogue1(int i) { return i >= 2 && i <= 16 && i % 2 == 0 ? (i - 2) / 2 : -1; }
constexpr int fs_epilogue0(int i) { return i >= 130 && i <= 142 && i % 2 == 0 ? (i - 130) / 2 : (i == 143 ? 7 : -1); }

template <int MI, bool STATS>
__global__ __launch_bounds__(256) void conv_fs64_kernel(const HaloArgs a)
{
    constexpr int TILE = 128 * MI, WPOS = 32 * MI, NLD = 4 * MI;   // a wavefront stages / stores WPOS rows: NLD 16-byte pieces per lane
    static_assert(64 * H_W_STRIDE <= F_RING_MAX * F_SLOT, "the filter passes through the ring's space");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char *ring = smem;                                   // F_RING_MAX * 144
    const int tid = threadIdx.x, lane = tid & 63;
    const int x = __builtin_amdgcn_readfirstlane(tid >> 6);
    unsigned char *strip = smem + F_RING_MAX * F_SLOT + x * (WPOS * F_SLOT);   // private: WPOS positions x 144 B
    const int frow = lane & 31, fk = lane >> 5;
    const int prow = lane >> 3, chunk = lane & 7;
    const __amdgpu_buffer_rsrc_t src_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.src, 0, a.src_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t out_rsrc = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, a.out_bytes, 0x00020000);

    const int tiles_per_block = (a.tiles + (int)gridDim.x - 1) / (int)gridDim.x;
    const int T0 = blockIdx.x * tiles_per_block;
    const int n = min(a.tiles, T0 + tiles_per_block) - T0;      // tiles of this block

    float ssum[8], ssq[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) ssum[e] = ssq[e] = 0.f;
    auto write_stats = [&]() {
        if (!STATS) return;
#pragma unroll
        for (int e = 0; e < 8; ++e)
#pragma unroll
            for (int o = 8; o < 64; o <<= 1) {
                ssum[e] += __shfl_xor(ssum[e], o, 64);
                ssq[e] += __shfl_xor(ssq[e], o, 64);
            }
        if (lane < 8) {
            float *r0 = a.stats + (size_t)(blockIdx.x * 4 + x) * 64 + lane * 8;
            float *r1 = r0 + (size_t)a.stats_rows * 64;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                r0[e] = ssum[e];
                r1[e] = ssq[e];
            }
        }
    };
    if (n <= 0) {                                                // uniform for the block: no barrier is skipped
        write_stats();                                           // zeros: every row of the buffer is written
        return;
    }

    const unsigned RING = (unsigned)(2 * TILE + 2 * a.halo);
    const int Q0 = T0 * TILE - a.halo;                           // padded position held by ring row 0
    // Byte offset of padded position q in the NHWC tensor (input and output have the same geometry), or out of
    // range; in two halves so that each fits between two MFMAs.
    unsigned so_img, so_rem;
    bool so_inside;
    auto src_offset_a = [&](int q) {
        so_inside = (unsigned)q < (unsigned)a.total_pos;
        const unsigned qq = so_inside ? (unsigned)q : 0u;
        so_img = (unsigned)(((unsigned long long)qq * a.magic_pi) >> 40);
        so_rem = qq - so_img * (unsigned)a.PI;
    };
    auto src_offset_b = [&]() -> unsigned {
        const unsigned hp = (unsigned)(((unsigned long long)so_rem * a.magic_pw) >> 40);
        const unsigned wp = so_rem - hp * (unsigned)a.PW;
        const bool ok = so_inside & (hp - 1u < (unsigned)a.H) & (wp - 1u < (unsigned)a.W);
        const unsigned off = (((so_img * a.H + (hp - 1u)) * a.W + (wp - 1u)) * 64u) * 2u;
        return ok ? off : H_OOB;
    };
    auto wrap = [&](unsigned s) -> unsigned { return min(s, s - RING); };   // s < 2*RING  ->  s mod RING

    bf16x8 wf[36][2];
    {
        // ---- requests first: the filter (whole block) and ring rows [0, TILE + 2*halo) (64 rows per wavefront and pass)
        u32x4 wtmp[18], v0[8], v1[8];
        const u32x4 *w = (const u32x4 *)a.wpk;
#pragma unroll
        for (int u = 0; u < 18; ++u) wtmp[u] = w[tid + 256 * u];
        const int rows0 = TILE + 2 * a.halo;                     // <= 384: at most two passes
        src_offset_a(Q0 + 64 * x + lane);
        const unsigned mine0 = src_offset_b();
        src_offset_a(Q0 + 256 + 64 * x + lane);
        const unsigned mine1 = src_offset_b();
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const unsigned o0 = (unsigned)__builtin_amdgcn_ds_bpermute((prow + 8 * u) * 4, (int)mine0) + (unsigned)(chunk * 16);
            const unsigned o1 = (unsigned)__builtin_amdgcn_ds_bpermute((prow + 8 * u) * 4, (int)mine1) + (unsigned)(chunk * 16);
            v0[u] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, o0, 0, 0);
            v1[u] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, 256 + 64 * x < rows0 ? o1 : H_OOB, 0, 0);
        }
        // ---- the filter through LDS into operand registers: wf[s][ni] = wpk[32*ni + frow][16*s + 8*fk .. + 7]
#pragma unroll
        for (int u = 0; u < 18; ++u) {
            const int i = tid + 256 * u, row = i / 72, vv = i - row * 72;
            *(u32x4 *)(smem + row * H_W_STRIDE + vv * 16) = wtmp[u];
        }
        lds_barrier();
        const unsigned char *wl = smem + frow * H_W_STRIDE + fk * 16;
#pragma unroll
        for (int s = 0; s < 36; ++s)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) wf[s][ni] = *(const bf16x8 *)(wl + ni * 32 * H_W_STRIDE + s * 32);
        // The first 32 steps' fragments (256 registers) are moved into the accumulation-register half of the file,
        // where the MFMAs read them directly; left to itself the compiler parks them there as spills and copies
        // eight registers back per step.
#pragma unroll
        for (int s = 0; s < F_AGPR_STEPS; ++s)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) asm volatile("" : "+a"(wf[s][ni]));
        lds_barrier();                                           // everyone has read the filter: the ring may be written
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int r = 64 * x + prow + 8 * u;
            *(u32x4 *)(ring + r * F_SLOT + chunk * 16) = v0[u];
            if (r + 256 < rows0) *(u32x4 *)(ring + (r + 256) * F_SLOT + chunk * 16) = v1[u];
        }
    }

    unsigned cs = 0;   // ring slot of row 0 of the tile being multiplied: (TILE * p) mod RING
    u32x4 st[NLD];     // input rows on their way from global memory to the ring
    unsigned offI[NLD], ooff[NLD];
    unsigned mineI = H_OOB, mineF = H_OOB;
    u32x4 sv[NLD];     // a tile's outputs on their way from the strip to global memory
    // the rows tile 1 needs beyond tile 0 are requested now and go to the ring during tile 0; from then on the rows
    // of tile p+2 are requested during tile p, so a request has a whole tile's time to come back from HBM
    {
        src_offset_a(Q0 + TILE + 2 * a.halo + WPOS * x + (lane & (WPOS - 1)));
        mineI = 1 < n ? src_offset_b() : H_OOB;
#pragma unroll
        for (int u = 0; u < NLD; ++u) {
            const unsigned o = (unsigned)__builtin_amdgcn_ds_bpermute((prow + 8 * u) * 4, (int)mineI) + (unsigned)(chunk * 16);
            st[u] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, o, 0, 0);
        }
    }

    f32x16 acc[2][MI];
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    lds_barrier();


    // acc[ni][mi][4g+j] is channel 32ni + 8g + 4fk + j of position 32mi + frow: piece e = 4*ni + g of position tile mi
    // converts four of them and writes 8 bytes of the strip
    auto epilogue_piece = [&](auto mic, auto ec) {
        constexpr int mi = decltype(mic)::value, ni = decltype(ec)::value >> 2, g = decltype(ec)::value & 3;
        bf16x4 pk;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) pk[jj] = (bf16_t)acc[ni][mi][g * 4 + jj];
        *(bf16x4 *)(strip + (mi * 32 + frow) * F_SLOT + (ni * 32 + g * 8 + fk * 4) * 2) = pk;
    };
    // statistics of stored outputs: one dword (two channels) of sv per call
    auto stats_piece = [&](auto ec) {
        constexpr int e2 = decltype(ec)::value, u = e2 >> 2, d = e2 & 3;
        const unsigned w = sv[u][d];
        const float lo = __builtin_bit_cast(float, w << 16), hi = __builtin_bit_cast(float, w & 0xFFFF0000u);
        ssum[2 * d] += lo;
        ssq[2 * d] += lo * lo;
        ssum[2 * d + 1] += hi;
        ssq[2 * d + 1] += hi * hi;
    };
    constexpr int NPAIR = 36 * MI, DIST = 4;   // input fragments are read DIST pairs (8 MFMAs) ahead

    for (int p = 0; p < n; ++p) {
        // ring row (before wrapping) of this lane's position of tile p, plus the halo: a tap adds its shift
        unsigned base[MI];
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) base[mi] = cs + (unsigned)(x * WPOS + mi * 32 + frow + a.halo);
        // first ring row (before wrapping) this lane writes for the next tile; kept as one value per tile so that the
        // eight row numbers are not carried across the loop as eight registers
        unsigned cbase = cs + (unsigned)(TILE + 2 * a.halo + WPOS * x + prow);
        asm volatile("" : "+v"(cbase));
        bf16x8 af[DIST + 1];
        unsigned ta[2][MI];   // fragment addresses of two taps in flight
        auto tap_addr = [&](int t, int mi) {
            ta[t & 1][mi] = __umul24(wrap(base[mi] + (unsigned)a.tapoff[t]), (unsigned)F_SLOT) + (unsigned)(fk * 16);
        };
        auto fetch = [&](auto pc) {
            constexpr int pair = decltype(pc)::value, step = fs_pair_step<MI>(pair), mi = fs_pair_mi<MI>(pair);
            af[pair % (DIST + 1)] = *(const bf16x8 *)(ring + ta[(step >> 2) & 1][mi] + (step & 3) * 32);
        };
        // index arithmetic of src_offset in five pieces (state in so_*)
        unsigned so_q, so_hp, so_wp;
        auto so1 = [&](int q) {
            so_inside = (unsigned)q < (unsigned)a.total_pos;
            so_q = so_inside ? (unsigned)q : 0u;
            so_img = (unsigned)(((unsigned long long)so_q * a.magic_pi) >> 40);
        };
        auto so2 = [&]() { so_rem = so_q - so_img * (unsigned)a.PI; };
        auto so3 = [&]() { so_hp = (unsigned)(((unsigned long long)so_rem * a.magic_pw) >> 40); };
        auto so4 = [&]() {
            so_wp = so_rem - so_hp * (unsigned)a.PW;
            so_inside = so_inside & (so_hp - 1u < (unsigned)a.H) & (so_wp - 1u < (unsigned)a.W);
        };
        auto so5 = [&]() -> unsigned {
            const unsigned off = (((so_img * a.H + (so_hp - 1u)) * a.W + (so_wp - 1u)) * 64u) * 2u;
            return so_inside ? off : H_OOB;
        };
        auto side = [&](auto mc) {
            constexpr FsAct act = fs_action<MI>(decltype(mc)::value);
            constexpr int k = act.kind, g = act.arg;
            if constexpr (k == F_TAP) tap_addr(g >> 1, g & 1);
            if constexpr (k == F_IA1) so1(Q0 + TILE * (p + 2) + 2 * a.halo + WPOS * x + (lane & (WPOS - 1)));
            if constexpr (k == F_IA2) so2();
            if constexpr (k == F_IB1) so3();
            if constexpr (k == F_IB2) so4();
            if constexpr (k == F_IB3) mineI = p + 2 < n ? so5() : H_OOB;
            if constexpr (k == F_IBP) {
#pragma unroll
                for (int u = g * 4; u < (g + 1) * 4 && u < NLD; ++u) offI[u] = (unsigned)__builtin_amdgcn_ds_bpermute((prow + 8 * u) * 4, (int)mineI);
            }
            if constexpr (k == F_CL) {
                // a row of the next tile: unwrapped row cs + TILE + 2*halo + ... (below 2*RING); after the block's last
                // tile these are rows nobody reads (this loop has no branches: every one costs an instruction refetch)
                const unsigned r = wrap(cbase + (unsigned)(8 * g));
                *(u32x4 *)(ring + __umul24(r, (unsigned)F_SLOT) + chunk * 16) = st[g];
                st[g] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, offI[g] + (unsigned)(chunk * 16), 0, 0);
            }
            // the outputs of the previous tile (in a block's first tile: stored nowhere, their offset is out of range)
            if constexpr (k == F_FA1) so1((T0 + p - 1) * TILE + WPOS * x + (lane & (WPOS - 1)));
            if constexpr (k == F_FA2) so2();
            if constexpr (k == F_FB1) so3();
            if constexpr (k == F_FB2) so4();
            if constexpr (k == F_FB3) mineF = p > 0 ? so5() : H_OOB;
        };
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) tap_addr(0, mi);
        tap_addr(1, 0);
        static_for<0, DIST>([&](auto pc) { fetch(pc); });
        static_for<0, 2 * NPAIR>([&](auto ic) {
            constexpr int i = decltype(ic)::value, pair = i >> 1, ni = i & 1;
            constexpr int step = fs_pair_step<MI>(pair), mi = fs_pair_mi<MI>(pair);
            if constexpr (ni == 0) {
                if constexpr (pair + DIST < NPAIR) fetch(std::integral_constant<int, pair + DIST>{});
                if constexpr (STATS && fs_out_count<MI>(pair) >= 0) {
                    static_for<0, (MI == 2 ? 1 : 4)>([&](auto dc) { stats_piece(std::integral_constant<int, fs_out_count<MI>(pair) + decltype(dc)::value>{}); });
                }
            } else {
                side(std::integral_constant<int, pair>{});
                if constexpr (fs_out_read<MI>(pair) >= 0) {
                    constexpr int g = fs_out_read<MI>(pair);
                    sv[g] = *(const u32x4 *)(strip + (prow + 8 * g) * F_SLOT + chunk * 16);
                    ooff[g] = (unsigned)__builtin_amdgcn_ds_bpermute((prow + 8 * g) * 4, (int)mineF);
                }
                if constexpr (fs_out_store<MI>(pair) >= 0) {
                    constexpr int g = fs_out_store<MI>(pair);
                    __builtin_amdgcn_raw_buffer_store_b128(sv[g], out_rsrc, ooff[g] + (unsigned)(chunk * 16), 0, 0);
                    if (STATS && ooff[g] >= H_OOB) sv[g] = u32x4{0u, 0u, 0u, 0u};   // padding positions are not stored and not counted
                }
            }
            if constexpr (MI == 2) {
                if constexpr (fs_epilogue1(i) >= 0) epilogue_piece(std::integral_constant<int, 1>{}, std::integral_constant<int, fs_epilogue1(i)>{});
                if constexpr (fs_epilogue0(i) >= 0) epilogue_piece(std::integral_constant<int, 0>{}, std::integral_constant<int, fs_epilogue0(i)>{});
            }
            __builtin_amdgcn_sched_barrier(0);
            acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[step][ni], af[pair % (DIST + 1)],
                                                                  step == 0 ? zero16 : acc[ni][mi], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        });
        if constexpr (MI == 1) static_for<0, 8>([&](auto ec) { epilogue_piece(std::integral_constant<int, 0>{}, ec); });
        cs = wrap(cs + (unsigned)TILE);
        lds_barrier();
    }
    // what is left: position tile 1 of the last tile, and the last tile's outputs
    if constexpr (MI == 2) static_for<0, 8>([&](auto ec) { epilogue_piece(std::integral_constant<int, 1>{}, ec); });
    {
        src_offset_a((T0 + n - 1) * TILE + WPOS * x + (lane & (WPOS - 1)));
        mineF = src_offset_b();
#pragma unroll
        for (int u = 0; u < NLD; ++u) {
            const unsigned o = (unsigned)__builtin_amdgcn_ds_bpermute((prow + 8 * u) * 4, (int)mineF) + (unsigned)(chunk * 16);
            const u32x4 v = *(const u32x4 *)(strip + (prow + 8 * u) * F_SLOT + chunk * 16);
            __builtin_amdgcn_raw_buffer_store_b128(v, out_rsrc, o, 0, 0);
            if (STATS) {
                const float live = o < H_OOB ? 1.f : 0.f;
                const bf16x8 vb = __builtin_bit_cast(bf16x8, v);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float f = live * (float)vb[e];
                    ssum[e] += f;
                    ssq[e] += f * f;
                }
            }
        }
    }
    write_stats();
}

}  // namespace

// True if the launch described by `a` is the shape this kernel covers.
bool halo64_applicable(int dtype, const IgemmArgs &a)
{
    if (dtype != NSK_BF16 || a.Cs != 64 || a.Ngemm != 64 || a.ntaps != 9 || a.Co != 64) return false;
    if (a.mult_h != 1 || a.mult_w != 1 || a.osh != 1 || a.osw != 1 || a.oa != 0 || a.ob != 0) return false;
    if (a.Hs != a.Ho || a.Ws != a.Wo || a.Mi != a.Ho || a.Mj != a.Wo) return false;
    if (HT + 2 * (a.Ws + 3) > H_MAX_IN) return false;
    for (int t = 0; t < 9; ++t) {
        const int eh = a.add_h + a.off_h[t], ew = a.add_w + a.off_w[t];
        if (eh < -1 || eh > 1 || ew < -1 || ew > 1) return false;
    }
    const long long pi = (long long)(a.Hs + 2) * (a.Ws + 2), total = pi * a.Nimg;
    if (total >= (1LL << 30) || total * pi >= (1LL << 40)) return false;   // exactness of the reciprocal division
    if ((unsigned long long)a.src_bytes >= H_OOB) return false;
    if (((uintptr_t)a.src | (uintptr_t)a.wpk | (uintptr_t)a.out) & 15) return false;
    return true;
}

namespace {
bool two_group(const IgemmArgs &g) { return 512 + 2 * (g.Ws + 3) <= P_RING_MAX && !hooks().halo_single; }
constexpr int kStatsGrid = 256;   // block count when statistics are requested: the row count must not depend on the device

// Which instance of the filter-stationary kernel takes the launch: 0 (none: accumulating launches keep the kernels
// above, which add the old values before the one rounding), else MI = positions per wavefront / 32.  The smaller
// tile is chosen where it fills the last round of tiles better (batch 64 at 56x56: 7 x 128 against 4 x 256 positions
// per block).  Depends on the geometry only, so that the planner and the launch agree.
int fs_choice(const IgemmArgs &g)
{
    if (g.accumulate || hooks().no_fs) return 0;
    const long long total = (long long)(g.Hs + 2) * (g.Ws + 2) * g.Nimg;
    const bool fits2 = 512 + 2 * (g.Ws + 3) <= F_RING_MAX, fits1 = 256 + 2 * (g.Ws + 3) <= F_RING_MAX;
    if (!fits1) return 0;
    const long long t2 = (total + 255) / 256, t1 = (total + 127) / 128;
    const long long cost2 = (t2 + kStatsGrid - 1) / kStatsGrid * 256, cost1 = (t1 + kStatsGrid - 1) / kStatsGrid * 128;
    if (!fits2) return 1;
    return cost1 * 100 < cost2 * 97 ? 1 : 2;
}
}  // namespace

// Rows of partial sums the forward launch writes (one per wavefront), 0 if this shape takes the kernel without a
// statistics epilogue.
int halo64_stats_rows(const IgemmArgs &g)
{
    if (g.accumulate) return 0;
    const int total = (g.Hs + 2) * (g.Ws + 2) * g.Nimg;
    const int mi = fs_choice(g);
    if (mi) {
        const int tiles = ceil_div(total, 128 * mi);
        return (tiles < kStatsGrid ? tiles : kStatsGrid) * 4;
    }
    if (!two_group(g)) return 0;
    const int tiles = ceil_div(total, HT);
    return (tiles < kStatsGrid ? tiles : kStatsGrid) * 8;
}

int launch_halo64(const IgemmArgs &g, hipStream_t stream)
{
    HaloArgs a{};
    a.src = g.src; a.wpk = g.wpk; a.out = g.out;
    a.N = g.Nimg; a.H = g.Hs; a.W = g.Ws;
    a.PW = g.Ws + 2; a.PI = (g.Hs + 2) * a.PW;
    a.total_pos = a.PI * g.Nimg;
    a.tiles = ceil_div(a.total_pos, HT);
    a.halo = a.PW + 1;
    a.magic_pi = ((1ULL << 40) + a.PI - 1) / a.PI;
    a.magic_pw = ((1ULL << 40) + a.PW - 1) / a.PW;
    a.src_bytes = g.src_bytes;
    a.out_bytes = g.src_bytes;   // same geometry: N*H*W*64 bf16
    a.accumulate = g.accumulate;
    a.stats = g.stats;
    a.stats_rows = g.stats_rows;
    for (int t = 0; t < 9; ++t) a.tapoff[t] = (g.add_h + g.off_h[t]) * a.PW + (g.add_w + g.off_w[t]);
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return NSK_ERR_HIP;
        cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    }
    const int want = g.stats ? kStatsGrid : cus;
    const int mi = fs_choice(g);
    if (mi) a.tiles = ceil_div(a.total_pos, 128 * mi);
    const int grid = a.tiles < want ? a.tiles : want;
    if (g.stats && g.stats_rows != grid * (mi ? 4 : 8)) return NSK_ERR_BAD_DESC;   // the planner and the launch disagree
    static bool attr_set = false;
    const int smem = H_MAX_IN * H_IN_STRIDE + 64 * H_W_STRIDE + 256 * 4 + H_MAX_IN * 4 + 4 * 32 * H_IN_STRIDE;
    const int smem_pp = P_RING_MAX * P_SLOT + 64 * H_W_STRIDE;
    const int smem_fs = F_RING_MAX * F_SLOT + 4 * 64 * F_SLOT;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)conv_halo64_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)conv_halo64_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)conv_halo64_pp_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_pp);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)conv_halo64_pp_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_pp);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)conv_fs64_kernel<1, false>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_fs);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)conv_fs64_kernel<1, true>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_fs);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)conv_fs64_kernel<2, false>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_fs);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)conv_fs64_kernel<2, true>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_fs);
        if (e != hipSuccess) {
            set_last_hip_error(e);
            return NSK_ERR_HIP;
        }
        attr_set = true;
    }
    if (mi) {
        if (mi == 1 && g.stats)
            hipLaunchKernelGGL((conv_fs64_kernel<1, true>), dim3(grid), dim3(256), smem_fs, stream, a);
        else if (mi == 1)
            hipLaunchKernelGGL((conv_fs64_kernel<1, false>), dim3(grid), dim3(256), smem_fs, stream, a);
        else if (g.stats)
            hipLaunchKernelGGL((conv_fs64_kernel<2, true>), dim3(grid), dim3(256), smem_fs, stream, a);
        else
            hipLaunchKernelGGL((conv_fs64_kernel<2, false>), dim3(grid), dim3(256), smem_fs, stream, a);
        return check_launch();
    }
    // the two-group kernel needs its ring (512 + 2*halo slots) to fit; wider images take the single-group kernel
    const bool pp = two_group(g);
    if (pp) {
        if (a.accumulate)
            hipLaunchKernelGGL(conv_halo64_pp_kernel<true>, dim3(grid), dim3(512), smem_pp, stream, a);
        else
            hipLaunchKernelGGL(conv_halo64_pp_kernel<false>, dim3(grid), dim3(512), smem_pp, stream, a);
    } else if (a.accumulate)
        hipLaunchKernelGGL(conv_halo64_kernel<true>, dim3(grid), dim3(256), smem, stream, a);
    else
        hipLaunchKernelGGL(conv_halo64_kernel<false>, dim3(grid), dim3(256), smem, stream, a);
    return check_launch();
}

}  // namespace nsk

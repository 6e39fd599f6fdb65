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
}  // namespace

// Rows of partial sums the forward launch writes (8 per block), 0 if this shape takes the kernel without a
// statistics epilogue.
int halo64_stats_rows(const IgemmArgs &g)
{
    if (!two_group(g) || g.accumulate) return 0;
    const int total = (g.Hs + 2) * (g.Ws + 2) * g.Nimg;
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
    const int grid = a.tiles < want ? a.tiles : want;
    if (g.stats && g.stats_rows != grid * 8) return NSK_ERR_BAD_DESC;   // the planner and the launch disagree
    static bool attr_set = false;
    const int smem = H_MAX_IN * H_IN_STRIDE + 64 * H_W_STRIDE + 256 * 4 + H_MAX_IN * 4 + 4 * 32 * H_IN_STRIDE;
    const int smem_pp = P_RING_MAX * P_SLOT + 64 * H_W_STRIDE;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)conv_halo64_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)conv_halo64_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)conv_halo64_pp_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_pp);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)conv_halo64_pp_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_pp);
        if (e != hipSuccess) {
            set_last_hip_error(e);
            return NSK_ERR_HIP;
        }
        attr_set = true;
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

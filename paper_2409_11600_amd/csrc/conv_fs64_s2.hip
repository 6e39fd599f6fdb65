// Backward-data of the bf16 3x3, stride 2, pad 1, 64 -> 64 channel layer (the strided layer of the bottleneck stage
// with 64-channel 3x3 filters; section "Experiments and Discussion" trains such residual networks): all four residue
// classes of the input gradient in ONE launch of a filter-stationary kernel.
//
// dx[2i+a][2j+b] for the residue class (a, b) receives dy[i + oh][j + ow] * w over the taps of that class only:
// one tap for (0,0), two for (0,1) and (1,0), four for (1,1), with offsets oh, ow in {0, 1}.  dy is addressed in
// flat coordinates of a grid padded by one row below and one column to the right ((Hs+1) x (Ws+1) per image, all
// images end to end), so a tap is one of the four constant shifts {0, 1, PW, PW+1}, positions outside the image load
// zeros through out-of-range buffer offsets, and a tile is 256 consecutive positions.  The layer is bound by the
// write of dx (four times the size of dy): what matters is that dy is read once, that the nine taps' products never
// leave the chip, and that the stores are whole 128-byte pixels.
//
// Structure as in the stride-1 filter-stationary kernel (conv_halo64.hip): four wavefronts, one per SIMD; each keeps
// ALL nine taps' filter fragments (four packed class filters, 36 reduction steps x 2 channel halves x 4 registers =
// 288) in registers for the life of the block, 256 of them accumulation registers that the MFMAs read directly; the
// dy fragments are the only LDS reads of the multiply loop (input ring of 2*256 + halo rows of 144 bytes).  A
// wavefront owns 64 positions (two position tiles of 32) x 64 channels.  Per tile it runs the four classes one after
// the other, each class position tile 0 first and then position tile 1, so that the accumulators of one position
// tile are converted to bf16 and written to LDS (a private strip, position-major, two strips in turn) while the
// MFMAs of the other run.  Everything else is cut into pieces of a few instructions that sit in front of single
// MFMAs of the fully unrolled loop (a compile-time schedule): reading a class's strip back and storing it to its
// pixels of dx, the index arithmetic, and the input rows for later tiles (requested a whole tile before they are
// written to the ring).  One LDS-only barrier per tile.
#include "nsk_internal.h"

namespace nsk {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr unsigned S2_OOB = 0xF0000000u;
constexpr int S2_SLOT = 144;             // bytes per ring row / strip row (64 bf16 + 16 pad: conflict-free fragment reads)
constexpr int S2_RING_MAX = 576;         // rows: 2*256 + halo, halo = Ws + 2 <= 64
constexpr int S2_W_STRIDE = 1168;        // bytes per filter row while the filter passes through LDS (9*64 bf16 + 16 pad)
constexpr int S2_AGPR_STEPS = 24;        // reduction steps whose filter fragments live in accumulation registers
constexpr int S2_TILE = 256, S2_WPOS = 64, S2_NLD = 8, S2_DIST = 4, S2_NPAIR = 72;

struct S2Args {
    const void *src;         // dy [N][Hs][Ws][64]
    void *out;               // dx [N][2*Hs][2*Ws][64]
    const void *wpk[4];      // packed class filters [64][ntaps][64], classes in the order (0,0), (0,1), (1,0), (1,1)
    unsigned oshift[4];      // byte offset of pixel (a, b) of a 2x2 output cell
    int N, Hs, Ws, PW, PI, total_pos, tiles, halo;
    unsigned long long magic_pi, magic_pw;
    unsigned src_bytes, out_bytes;
};

// ---- the compile-time schedule -----------------------------------------------------------------------------------
// Pairs (two MFMAs on one dy fragment) of a tile: class c occupies pairs [P0[c], P0[c] + 2*L[c]), position tile 0
// first; L = 4 * taps = 4, 8, 8, 16 reduction steps.
constexpr int s2_class(int pair) { return pair < 8 ? 0 : pair < 24 ? 1 : pair < 40 ? 2 : 3; }
constexpr int s2_p0(int c) { return c == 0 ? 0 : c == 1 ? 8 : c == 2 ? 24 : 40; }
constexpr int s2_len(int c) { return c == 0 ? 4 : c == 3 ? 16 : 8; }
constexpr int s2_s0(int c) { return c == 0 ? 0 : c == 1 ? 4 : c == 2 ? 12 : 20; }     // first reduction step of the class
constexpr int s2_mi(int pair) { return pair - s2_p0(s2_class(pair)) >= s2_len(s2_class(pair)) ? 1 : 0; }
constexpr int s2_lstep(int pair) { return pair - s2_p0(s2_class(pair)) - s2_mi(pair) * s2_len(s2_class(pair)); }
constexpr int s2_gstep(int pair) { return s2_s0(s2_class(pair)) + s2_lstep(pair); }
// shift of tap t of class c as 2*oh + ow (the order in which the classes' taps are packed: filter rows r ascending,
// then s ascending, which is oh descending, then ow descending)
constexpr int s2_shift(int c, int t) { return c == 0 ? 0 : c == 1 ? (t == 0 ? 1 : 0) : c == 2 ? (t == 0 ? 2 : 0) : 3 - t; }
constexpr int s2_pair_shift(int pair) { return s2_shift(s2_class(pair), s2_lstep(pair) >> 2); }
// Conversion pieces (eight per class and position tile: piece e = 4*ni + g) in front of MFMA i; a class's position
// tile 0 is converted while its position tile 1 is multiplied, position tile 1 while the next class starts.  The
// first window (class 0, position tile 0) is only eight MFMAs long, so two of its slots take two pieces; the last one
// (class 3, position tile 1) lies in the NEXT tile.  Returns the first piece of (c, mi) in slot i and their count.
struct S2Epi { int first, count; };
constexpr S2Epi s2_epi(int c, int mi, int i)
{
    if (c == 0 && mi == 0) {
        switch (i) {
        case 10: return {0, 1}; case 11: return {1, 1}; case 12: return {2, 2}; case 13: return {4, 1};
        case 14: return {5, 1}; case 15: return {6, 2};
        default: return {0, 0};
        }
    }
    const int start = c == 0 ? 18 : c == 1 ? (mi == 0 ? 34 : 50) : c == 2 ? (mi == 0 ? 66 : 82) : (mi == 0 ? 114 : 0);
    return i >= start && i < start + 8 ? S2Epi{i - start, 1} : S2Epi{0, 0};
}
// Output pipeline: vector g (0..7) of class c is read back from its strip in the side slot of pair s2_out_read and
// stored two pairs later; class 3 leaves during the next tile.
constexpr int s2_out_base(int c) { return c == 0 ? 13 : c == 1 ? 29 : c == 2 ? 45 : 4; }
// Side actions by pair (slot in front of the pair's second MFMA)
enum { S2_NONE, S2_FA1, S2_FA2, S2_FB1, S2_FB2, S2_FB3, S2_IA1, S2_IA2, S2_IB1, S2_IB2, S2_IB3, S2_IBP, S2_CL };
struct S2Act { int kind, arg; };
constexpr S2Act s2_action(int m)
{
    switch (m) {
    case 0: return {S2_FA1, 0}; case 1: return {S2_FA2, 0}; case 2: return {S2_FB1, 0}; case 3: return {S2_FB2, 0}; case 12: return {S2_FB3, 0};
    case 21: return {S2_IA1, 0}; case 22: return {S2_IA2, 0}; case 23: return {S2_IB1, 0}; case 24: return {S2_IB2, 0}; case 25: return {S2_IB3, 0};
    case 26: return {S2_IBP, 0}; case 27: return {S2_IBP, 1};
    case 37: return {S2_CL, 0}; case 38: return {S2_CL, 1}; case 39: return {S2_CL, 2}; case 40: return {S2_CL, 3};
    case 41: return {S2_CL, 4}; case 42: return {S2_CL, 5}; case 43: return {S2_CL, 6}; case 44: return {S2_CL, 7};
    default: return {S2_NONE, 0};
    }
}

__global__ __launch_bounds__(256) void conv_fs64_dgrad_s2_kernel(const S2Args a)
{
    constexpr int TILE = S2_TILE, WPOS = S2_WPOS, NLD = S2_NLD, DIST = S2_DIST, NPAIR = S2_NPAIR;
    static_assert(64 * S2_W_STRIDE <= S2_RING_MAX * S2_SLOT, "the filter passes through the ring's space");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char *ring = smem;                                   // S2_RING_MAX * 144
    const int tid = threadIdx.x, lane = tid & 63;
    const int x = __builtin_amdgcn_readfirstlane(tid >> 6);
    // two private strips of WPOS positions x 144 B per wavefront: classes 0 and 2 use strip 0, classes 1 and 3 strip 1
    unsigned char *strip0 = smem + S2_RING_MAX * S2_SLOT + x * (2 * WPOS * S2_SLOT);
    const int frow = lane & 31, fk = lane >> 5;
    const int prow = lane >> 3, chunk = lane & 7;
    const __amdgpu_buffer_rsrc_t src_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.src, 0, a.src_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t out_rsrc = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, a.out_bytes, 0x00020000);

    const int tiles_per_block = (a.tiles + (int)gridDim.x - 1) / (int)gridDim.x;
    const int T0 = blockIdx.x * tiles_per_block;
    const int n = min(a.tiles, T0 + tiles_per_block) - T0;      // tiles of this block
    if (n <= 0) return;                                          // uniform for the block: no barrier is skipped

    const unsigned RING = (unsigned)(2 * TILE + a.halo);
    const int Q0 = T0 * TILE;                                    // flat position held by ring row 0
    // Position q -> (image, i, j) in five small pieces (state in so_*); then either the byte offset of dy[i][j] or
    // of the output cell dx[2i][2j], out of range for padding positions.
    unsigned so_q, so_img, so_rem, so_i, so_j;
    bool so_ok;
    auto so1 = [&](int q) {
        so_ok = (unsigned)q < (unsigned)a.total_pos;
        so_q = so_ok ? (unsigned)q : 0u;
        so_img = (unsigned)(((unsigned long long)so_q * a.magic_pi) >> 40);
    };
    auto so2 = [&]() { so_rem = so_q - so_img * (unsigned)a.PI; };
    auto so3 = [&]() { so_i = (unsigned)(((unsigned long long)so_rem * a.magic_pw) >> 40); };
    auto so4 = [&]() {
        so_j = so_rem - so_i * (unsigned)a.PW;
        so_ok = so_ok & (so_i < (unsigned)a.Hs) & (so_j < (unsigned)a.Ws);
    };
    auto so5_src = [&]() -> unsigned {
        const unsigned off = (((so_img * a.Hs + so_i) * a.Ws + so_j) * 64u) * 2u;
        return so_ok ? off : S2_OOB;
    };
    auto so5_out = [&]() -> unsigned {
        const unsigned off = (((so_img * (2u * a.Hs) + 2u * so_i) * (2u * a.Ws) + 2u * so_j) * 64u) * 2u;
        return so_ok ? off : S2_OOB;
    };
    auto src_offset = [&](int q) -> unsigned {
        so1(q);
        so2();
        so3();
        so4();
        return so5_src();
    };
    auto wrap = [&](unsigned s) -> unsigned { return min(s, s - RING); };   // s < 2*RING  ->  s mod RING

    bf16x8 wf[36][2];
    {
        // ---- requests first: the four class filters (whole block: 64 rows x 72 vectors) and ring rows [0, TILE + halo)
        u32x4 wtmp[18], v0[8], v1[8];
#pragma unroll
        for (int u = 0; u < 18; ++u) {
            const int i = tid + 256 * u, row = i / 72, vv = i - row * 72, gt = vv >> 3, ch = vv & 7;
            // global tap gt -> class (taps 1, 2, 2, 4) and tap within the class
            const int c = (gt >= 1) + (gt >= 3) + (gt >= 5), tl = gt - (c == 0 ? 0 : c == 1 ? 1 : c == 2 ? 3 : 5);
            const int nt = c == 0 ? 1 : c == 3 ? 4 : 2;
            const unsigned char *w = (const unsigned char *)(c == 0 ? a.wpk[0] : c == 1 ? a.wpk[1] : c == 2 ? a.wpk[2] : a.wpk[3]);
            wtmp[u] = *(const u32x4 *)(w + ((row * nt + tl) * 64 + ch * 8) * 2);
        }
        const int rows0 = TILE + a.halo;                         // <= 320: two passes of 4 x 64 rows
        const unsigned mine0 = src_offset(Q0 + 64 * x + lane);
        const unsigned mine1 = src_offset(Q0 + 256 + 64 * x + lane);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const unsigned o0 = (unsigned)__builtin_amdgcn_ds_bpermute((prow + 8 * u) * 4, (int)mine0) + (unsigned)(chunk * 16);
            const unsigned o1 = (unsigned)__builtin_amdgcn_ds_bpermute((prow + 8 * u) * 4, (int)mine1) + (unsigned)(chunk * 16);
            v0[u] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, o0, 0, 0);
            v1[u] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, 256 + 64 * x < rows0 ? o1 : S2_OOB, 0, 0);
        }
        // ---- the filters through LDS into operand registers: wf[s][ni] = (row 32*ni + frow, reduction indices 16*s + 8*fk .. + 7)
#pragma unroll
        for (int u = 0; u < 18; ++u) {
            const int i = tid + 256 * u, row = i / 72, vv = i - row * 72;
            *(u32x4 *)(smem + row * S2_W_STRIDE + vv * 16) = wtmp[u];
        }
        lds_barrier();
        const unsigned char *wl = smem + frow * S2_W_STRIDE + fk * 16;
#pragma unroll
        for (int s = 0; s < 36; ++s)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) wf[s][ni] = *(const bf16x8 *)(wl + ni * 32 * S2_W_STRIDE + s * 32);
        // (see conv_halo64.hip: pinned once into accumulation registers, where the MFMAs read them directly)
#pragma unroll
        for (int s = 0; s < S2_AGPR_STEPS; ++s)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) asm volatile("" : "+a"(wf[s][ni]));
        lds_barrier();                                           // everyone has read the filters: the ring may be written
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int r = 64 * x + prow + 8 * u;
            *(u32x4 *)(ring + r * S2_SLOT + chunk * 16) = v0[u];
            if (r + 256 < rows0) *(u32x4 *)(ring + (r + 256) * S2_SLOT + chunk * 16) = v1[u];
        }
    }

    unsigned cs = 0;   // ring slot of row 0 of the tile being multiplied: (TILE * p) mod RING
    u32x4 st[NLD];     // input rows on their way from global memory to the ring
    unsigned offI[NLD];
    unsigned mineI = S2_OOB, mineF = S2_OOB, mineF_prev = S2_OOB;
    u32x4 sv[NLD];     // outputs on their way from a strip to global memory
    unsigned ooff[NLD];
    // the rows tile 1 needs beyond tile 0 are requested now and go to the ring during tile 0; from then on the rows
    // of tile p+2 are requested during tile p
    {
        mineI = src_offset(Q0 + TILE + a.halo + WPOS * x + lane);
        if (!(1 < n)) mineI = S2_OOB;
#pragma unroll
        for (int u = 0; u < NLD; ++u) {
            const unsigned o = (unsigned)__builtin_amdgcn_ds_bpermute((prow + 8 * u) * 4, (int)mineI) + (unsigned)(chunk * 16);
            st[u] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, o, 0, 0);
        }
    }

    f32x16 acc[2][2];
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    lds_barrier();

    // acc[ni][mi][4g+j] is channel 32ni + 8g + 4fk + j of position 32mi + frow: piece e = 4*ni + g of position tile mi
    // converts four of them and writes 8 bytes of class c's strip
    auto epilogue_piece = [&](auto cc, auto mic, auto ec) {
        constexpr int c = decltype(cc)::value, mi = decltype(mic)::value, ni = decltype(ec)::value >> 2, g = decltype(ec)::value & 3;
        bf16x4 pk;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) pk[jj] = (bf16_t)acc[ni][mi][g * 4 + jj];
        *(bf16x4 *)(strip0 + (c & 1) * (WPOS * S2_SLOT) + (mi * 32 + frow) * S2_SLOT + (ni * 32 + g * 8 + fk * 4) * 2) = pk;
    };
    auto out_read = [&](auto cc, auto gc, unsigned mine) {      // vector g of class c: strip -> registers, and its byte offset
        constexpr int c = decltype(cc)::value, g = decltype(gc)::value;
        sv[g] = *(const u32x4 *)(strip0 + (c & 1) * (WPOS * S2_SLOT) + (prow + 8 * g) * S2_SLOT + chunk * 16);
        ooff[g] = (unsigned)__builtin_amdgcn_ds_bpermute((prow + 8 * g) * 4, (int)mine);
    };
    auto out_store = [&](auto cc, auto gc) {
        constexpr int c = decltype(cc)::value, g = decltype(gc)::value;
        // (an out-of-range marker stays out of range after the small offsets are added)
        __builtin_amdgcn_raw_buffer_store_b128(sv[g], out_rsrc, ooff[g] + a.oshift[c] + (unsigned)(chunk * 16), 0, 0);
    };

    for (int p = 0; p < n; ++p) {
        // LDS addresses of this lane's dy fragments of tile p for the four shifts and the two position tiles
        unsigned ta[4][2];
#pragma unroll
        for (int sh = 0; sh < 4; ++sh)
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) {
                const unsigned r = wrap(cs + (unsigned)(x * WPOS + mi * 32 + frow + (sh >> 1) * a.PW + (sh & 1)));
                ta[sh][mi] = __umul24(r, (unsigned)S2_SLOT) + (unsigned)(fk * 16);
            }
        // first ring row (before wrapping) this lane writes for the next tile (one value per tile: see conv_halo64.hip)
        unsigned cbase = cs + (unsigned)(TILE + a.halo + WPOS * x + prow);
        asm volatile("" : "+v"(cbase));
        bf16x8 af[DIST + 1];
        auto fetch = [&](auto pc) {
            constexpr int pair = decltype(pc)::value;
            af[pair % (DIST + 1)] = *(const bf16x8 *)(ring + ta[s2_pair_shift(pair)][s2_mi(pair)] + (s2_lstep(pair) & 3) * 32);
        };
        auto side = [&](auto mc) {
            constexpr S2Act act = s2_action(decltype(mc)::value);
            constexpr int k = act.kind, g = act.arg;
            if constexpr (k == S2_FA1) so1((T0 + p) * TILE + WPOS * x + lane);
            if constexpr (k == S2_IA1) so1(Q0 + TILE * (p + 2) + a.halo + WPOS * x + lane);
            if constexpr (k == S2_FA2 || k == S2_IA2) so2();
            if constexpr (k == S2_FB1 || k == S2_IB1) so3();
            if constexpr (k == S2_FB2 || k == S2_IB2) so4();
            if constexpr (k == S2_FB3) mineF = so5_out();
            if constexpr (k == S2_IB3) mineI = p + 2 < n ? so5_src() : S2_OOB;
            if constexpr (k == S2_IBP) {
#pragma unroll
                for (int u = g * 4; u < (g + 1) * 4; ++u) offI[u] = (unsigned)__builtin_amdgcn_ds_bpermute((prow + 8 * u) * 4, (int)mineI);
            }
            if constexpr (k == S2_CL) {
                // a row of the next tile (after the block's last tile: rows nobody reads; no branch in this loop)
                const unsigned r = wrap(cbase + (unsigned)(8 * g));
                *(u32x4 *)(ring + __umul24(r, (unsigned)S2_SLOT) + chunk * 16) = st[g];
                st[g] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, offI[g] + (unsigned)(chunk * 16), 0, 0);
            }
        };
        static_for<0, DIST>([&](auto pc) { fetch(pc); });
        static_for<0, 2 * NPAIR>([&](auto ic) {
            constexpr int i = decltype(ic)::value, pair = i >> 1, ni = i & 1;
            constexpr int mi = s2_mi(pair), step = s2_gstep(pair);
            if constexpr (ni == 0) {
                if constexpr (pair + DIST < NPAIR) fetch(std::integral_constant<int, pair + DIST>{});
            } else {
                side(std::integral_constant<int, pair>{});
                // output pipeline: classes 0..2 of this tile, class 3 of the previous one
                static_for<0, 4>([&](auto cc) {
                    constexpr int oc = decltype(cc)::value, rel = pair - s2_out_base(oc);
                    // (in a block's first tile class 3 "of the previous tile" reads an unwritten strip and stores it at
                    // mineF_prev = out of range, i.e. nowhere)
                    if constexpr (rel >= 0 && rel < 8) out_read(cc, std::integral_constant<int, rel>{}, oc < 3 ? mineF : mineF_prev);
                    if constexpr (rel >= 2 && rel < 10) out_store(cc, std::integral_constant<int, rel - 2>{});
                });
            }
            // conversion pieces scheduled in front of this MFMA
            static_for<0, 4>([&](auto cc) {
                static_for<0, 2>([&](auto mic) {
                    constexpr S2Epi e = s2_epi(decltype(cc)::value, decltype(mic)::value, i);
                    if constexpr (e.count > 0) {
                        static_for<0, e.count>([&](auto kc) { epilogue_piece(cc, mic, std::integral_constant<int, e.first + decltype(kc)::value>{}); });
                    }
                });
            });
            __builtin_amdgcn_sched_barrier(0);
            acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[step][ni], af[pair % (DIST + 1)],
                                                                  s2_lstep(pair) == 0 ? zero16 : acc[ni][mi], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        });
        mineF_prev = mineF;
        cs = wrap(cs + (unsigned)TILE);
        lds_barrier();
    }
    // what is left: position tile 1 of class 3 of the last tile, and that class's outputs
    static_for<0, 8>([&](auto ec) { epilogue_piece(std::integral_constant<int, 3>{}, std::integral_constant<int, 1>{}, ec); });
    static_for<0, 8>([&](auto gc) { out_read(std::integral_constant<int, 3>{}, gc, mineF_prev); });
    static_for<0, 8>([&](auto gc) { out_store(std::integral_constant<int, 3>{}, gc); });
}


// ---------------------------------------------------------------------------------------------------------------------
// FORWARD of the same layer (3x3, stride 2, pad 1, 64 -> 64, even extents).  The input splits into four parity planes,
// plane (a, b) = x[2I-1+a][2J-1+b]; output position (I, J) reads plane (a, b) at (I + dI, J + dJ) with
//   filter row r = 0, 1, 2  ->  (a, dI) = (0, 0), (1, 0), (0, 1)   and the same for columns,
// so in flat coordinates of a (P+1) x (Q+1) grid every tap is one plane and one of the shifts {0, 1, PW, PW+1}: the
// stride disappears.  A pixel of a plane is 128 contiguous bytes of x, so a plane is staged like any other tensor, by
// byte offset per row, in whole cache lines.  Each plane has an input ring of its own, sized for the shifts that
// reach it (halo PW+1, PW, 1 and 0 rows for planes (0,0), (0,1), (1,0), (1,1)): 4 x 2 x 128 + 2*PW + 2 rows.
//
// Four wavefronts, the nine taps' filter fragments in registers, a tile of 128 positions (32 per wavefront, two
// MFMAs per input fragment), one LDS-only barrier per tile.  The layer reads four input pixels per output pixel: it
// is bound by memory, and next to that by the NUMBER of instructions per tile (with one wavefront per SIMD an MFMA
// hides only a handful of other instructions of the same wavefront):
//   * ring rows are 128 bytes with 16 bytes of padding after every second row (row r at (r/2)*272 + (r%2)*128):
//     fragment reads are conflict-free without a swizzle, so the four reduction steps of a tap are immediate offsets
//     of one address register, and advancing any address by a tile is an add and a wrap;
//   * every address (nine taps, sixteen staging pieces) lives in a register and is advanced in place;
//   * one division per lane and tile yields the offsets of all four planes (carries instead of a division each)
//     and, two tiles later, of the outputs;
//   * plane (1,1) is only reached by the centre tap, without a shift: its rows are private to the wavefront that
//     stages them, so the rows a tile has just consumed serve as the strip through which that wavefront turns its
//     accumulators into whole output pixels (no LDS beyond the rings).
// Input rows are requested two tiles ahead of their use (a tile in registers, a tile in the ring), outputs are
// converted after a tile's last MFMA and stored (and counted for the batch-norm statistics) during the next tile.
constexpr int F2_TILE = 128, F2_WPOS = 32, F2_NPAIR = 36, F2_DIST = 4;
constexpr int F2_PAIR_BYTES = 272;       // two ring rows and their padding
constexpr int F2_MAX_PW = 88;            // grid width (Q + 1) the rings hold: 4*256 + 2*PW + 3 rows <= 160 KB
constexpr int F2_AGPR_STEPS = 28;        // 224 accumulation registers of filter next to the 32 accumulators
constexpr int F2_STATS_GRID = 256;       // block count when statistics are requested (independent of the device)

struct F2Args {
    const void *src, *wpk;   // x [N][H][W][64]; packed filter [64][9][64], taps in (r, s) order
    void *out;               // y [N][P][Q][64]
    float *stats;            // nullptr, or partial sums of the stored output: 4 rows per block
    int stats_rows;
    int N, H, W, P, Q, PW, PR, PI, total_pos, tiles;
    unsigned img_bytes, row2_bytes;   // H*W*128 and 2*W*128: x bytes per image and per two rows
    unsigned long long magic_pi, magic_pw;
    unsigned src_bytes, out_bytes;
};

// tap t = 3r + s  ->  plane 2a + b and shift 2*dI + dJ
constexpr int f2_plane(int t) { return ((t / 3) == 1 ? 2 : 0) + ((t % 3) == 1 ? 1 : 0); }
constexpr int f2_shift(int t) { return ((t / 3) == 2 ? 2 : 0) + ((t % 3) == 2 ? 1 : 0); }
// rows a tile needs beyond its own 128 in plane c: (0,0): PW+1, (0,1): PW, (1,0): 1, (1,1): 0
__device__ __host__ constexpr int f2_halo(int c, int PW) { return c == 0 ? PW + 1 : c == 1 ? PW : c == 2 ? 1 : 0; }
__device__ __host__ constexpr int f2_ring_rows(int c, int PW) { return (2 * F2_TILE + f2_halo(c, PW) + 1) & ~1; }
__host__ constexpr int f2_lds_bytes(int PW)
{
    return (f2_ring_rows(0, PW) + f2_ring_rows(1, PW) + f2_ring_rows(2, PW) + f2_ring_rows(3, PW)) / 2 * F2_PAIR_BYTES;
}

// Order of the 16 input pieces (piece = plane c, rows 8u .. 8u+7 of a wavefront's 32): the two pixels of a 256-byte
// pair of x (planes (a,1) at a position and (a,0) at the next one for a = 0, planes (1,1) and (1,0) for a = 1) are
// requested one after the other
constexpr int f2_piece_c(int j) { return (j >> 3) == 0 ? ((j & 1) == 0 ? 1 : 0) : ((j & 1) == 0 ? 3 : 2); }
constexpr int f2_piece_u(int j) { return (j >> 1) & 3; }

// The compile-time schedule of a tile.  With one wavefront per SIMD an MFMA (32 clocks) hides about six independent
// or four dependent instructions of the same wavefront and no more, so the side work is spread over the 72 slots in
// front of the MFMAs a few instructions at a time.  Slot 2m is in front of the first MFMA of pair m (it also holds the
// request of the input fragment four pairs ahead), slot 2m+1 in front of the second.
enum { F2_NONE, F2_IA1, F2_IA2, F2_IA3, F2_IP, F2_OR, F2_OS, F2_ST, F2_TAPU, F2_CLW, F2_CLA };
struct F2Act { int kind, arg; };
constexpr F2Act f2_action(int slot)
{
    const int m = slot >> 1;
    if (m >= 14 && m < 30) return {(slot & 1) ? F2_CLA : F2_CLW, m - 14};   // input piece m - 14: commit and reload | advance
    switch (slot) {
    // input offsets of tile p+2 (a division per lane, then one plane at a time; the first pieces are planes 1, 0)
    case 1: return {F2_IA1, 0}; case 7: return {F2_IA2, 0}; case 13: return {F2_IA3, 0};
    case 19: return {F2_IP, 1}; case 25: return {F2_IP, 0}; case 22: return {F2_IP, 3}; case 26: return {F2_IP, 2};
    // output vector g of tile p-1: strip -> registers, store, statistics in two halves
    case 3: return {F2_OR, 0}; case 5: return {F2_OS, 0}; case 6: return {F2_ST, 0}; case 8: return {F2_ST, 1};
    case 9: return {F2_OR, 1}; case 11: return {F2_OS, 1}; case 12: return {F2_ST, 2}; case 14: return {F2_ST, 3};
    case 15: return {F2_OR, 2}; case 17: return {F2_OS, 2}; case 18: return {F2_ST, 4}; case 20: return {F2_ST, 5};
    case 21: return {F2_OR, 3}; case 23: return {F2_OS, 3}; case 24: return {F2_ST, 6}; case 27: return {F2_ST, 7};
    // a tap's address moves on to the next tile once its last fragment has been requested
    case 61: return {F2_TAPU, 0}; case 63: return {F2_TAPU, 1}; case 64: return {F2_TAPU, 2}; case 65: return {F2_TAPU, 3};
    case 66: return {F2_TAPU, 4}; case 67: return {F2_TAPU, 5}; case 68: return {F2_TAPU, 6}; case 69: return {F2_TAPU, 7};
    case 70: return {F2_TAPU, 8};
    default: return {F2_NONE, 0};
    }
}
// LDS access by address (a number of bytes from the start of the workgroup's LDS) and an index in units of T
template <typename T>
__device__ inline T lds_get(unsigned addr, int idx)
{
    typedef T __attribute__((address_space(3))) LT;
    return ((const LT *)(size_t)addr)[idx];
}
template <typename T>
__device__ inline void lds_put(unsigned addr, int idx, const T &v)
{
    typedef T __attribute__((address_space(3))) LT;
    ((LT *)(size_t)addr)[idx] = v;
}

template <bool STATS>
__global__ __launch_bounds__(256) void conv_fs64_fwd_s2_kernel(const F2Args a)
{
    constexpr int TILE = F2_TILE, WPOS = F2_WPOS, NPAIR = F2_NPAIR, DIST = F2_DIST;
    constexpr unsigned ADV = TILE / 2 * F2_PAIR_BYTES;          // LDS bytes of a tile's rows
    // The tile loop addresses LDS with plain 32-bit numbers kept in registers: the start of the allocation goes into
    // them once, here, and no access adds a base.
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const int tid = threadIdx.x, lane = tid & 63;
    const int x = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int frow = lane & 31, fk = lane >> 5;
    const int prow = lane >> 3, chunk = lane & 7;
    const unsigned chunk16 = (unsigned)chunk * 16u;
    const __amdgpu_buffer_rsrc_t src_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.src, 0, a.src_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t out_rsrc = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, a.out_bytes, 0x00020000);
    unsigned rbase[4], rsize[4], rend[4];
    {
        unsigned at = lds0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            rbase[c] = at;
            rsize[c] = (unsigned)(f2_ring_rows(c, a.PW) / 2 * F2_PAIR_BYTES);
            at += rsize[c];
            rend[c] = at;
        }
    }
    auto row_addr = [&](int c, unsigned r) -> unsigned { return rbase[c] + (r >> 1) * (unsigned)F2_PAIR_BYTES + (r & 1u) * 128u; };
    // an address of ring c one tile later (ring sizes are whole row pairs and a tile is 64 of them)
    auto advance = [&](unsigned addr, int c) -> unsigned {
        const unsigned t = addr + ADV;
        return t >= rend[c] ? t - rsize[c] : t;
    };

    const int tiles_per_block = (a.tiles + (int)gridDim.x - 1) / (int)gridDim.x;
    const int T0 = blockIdx.x * tiles_per_block;
    const int n = min(a.tiles, T0 + tiles_per_block) - T0;      // tiles of this block

    float ssum[8], ssq[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) ssum[e] = ssq[e] = 0.f;
    // lane (prow, chunk) has counted channels 8*chunk .. 8*chunk+7 of the rows it stored: add up over prow, one row
    // of partial sums per wavefront
    auto write_stats = [&]() {
        if constexpr (STATS) {
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
        }
    };
    if (n <= 0) {                                                // uniform for the block: no barrier is skipped
        write_stats();                                           // zeros: every row of the buffer is written
        return;
    }
    const int Q0 = T0 * TILE;                                    // flat position held by row 0 of every ring

    // Position q -> (image, I, J) in small pieces (state in so_*).  so_q keeps the unclamped position; a tile that
    // does not exist is handed in as position 2^30, beyond every grid this kernel takes (no branch in the tile loop).
    // so_src is the byte offset of x[2I-1][2J-1] (possibly outside x: only sums with a plane's own offset are used).
    unsigned so_q, so_img, so_rem, so_i, so_j, so_src, so_out;
    auto so1 = [&](int q) {
        so_q = (unsigned)q;
        const unsigned qc = so_q < (unsigned)a.total_pos ? so_q : 0u;
        so_img = (unsigned)(((unsigned long long)qc * a.magic_pi) >> 40);
        so_rem = qc - so_img * (unsigned)a.PI;
    };
    auto so2 = [&]() {
        so_i = (unsigned)(((unsigned long long)so_rem * a.magic_pw) >> 40);
        so_j = so_rem - so_i * (unsigned)a.PW;
    };
    auto so3 = [&]() {
        const unsigned t = so_img * a.img_bytes + so_i * a.row2_bytes;      // x[img][2I][0]; a quarter of it is y[img][I][0]
        so_src = t + so_j * 256u - (unsigned)((a.W + 1) * 128);
        const bool ok = (so_q < (unsigned)a.total_pos) & (so_i < (unsigned)a.P) & (so_j < (unsigned)a.Q);
        so_out = ok ? (t >> 2) + so_j * 128u : S2_OOB;
    };
    // Byte offset of the plane-c pixel of the position (di rows, dj columns) after the one just divided (carries into
    // the next grid row and the next image instead of a division per plane), out of range where that pixel does not
    // exist
    auto plane_off = [&](int c, int di, int dj) -> unsigned {
        const int pa = c >> 1, pb = c & 1;
        unsigned j = so_j + (unsigned)dj, i = so_i + (unsigned)di;
        unsigned off = so_src + (unsigned)(dj * 256 + (pa * a.W + pb) * 128) + (unsigned)di * a.row2_bytes;
        if (dj) {
            const bool cj = j >= (unsigned)a.PW;
            j = cj ? j - (unsigned)a.PW : j;
            off += cj ? a.row2_bytes - (unsigned)(a.PW * 256) : 0u;
            i += cj ? 1u : 0u;
        }
        if (di || dj) {
            const bool ci = i >= (unsigned)a.PR;
            i = ci ? i - (unsigned)a.PR : i;
            off += ci ? a.img_bytes - (unsigned)a.PR * a.row2_bytes : 0u;
        }
        const bool okh = pa ? i < (unsigned)a.P : i >= 1u, okw = pb ? j < (unsigned)a.Q : j >= 1u;
        const bool ok = (so_q + (unsigned)(di * a.PW + dj) < (unsigned)a.total_pos) & okh & okw;
        return ok ? off : S2_OOB;
    };
    auto plane_off_halo = [&](int c) -> unsigned { return plane_off(c, c < 2 ? 1 : 0, c == 0 || c == 2 ? 1 : 0); };

    bf16x8 wf[36][2];
    u32x4 st[16];      // input rows on their way from global memory to the rings: piece 4*c + u of plane c
    unsigned fq[3];    // output offsets of this lane's row of the previous, the current and the next tile
    fq[0] = S2_OOB;
    {
        // ---- requests first: the filter (whole block: 64 rows x 72 vectors) and, per plane, ring rows [0, TILE + halo)
        // in passes of 4 wavefronts x 32 rows (at most two passes: TILE + halo <= 256)
        u32x4 wtmp[18], v[2][16];
        const u32x4 *w = (const u32x4 *)a.wpk;
#pragma unroll
        for (int u = 0; u < 18; ++u) wtmp[u] = w[tid + 256 * u];
#pragma unroll
        for (int ps = 0; ps < 2; ++ps) {
            so1(Q0 + TILE * ps + WPOS * x + (lane & 31));
            so2();
            so3();
            if (ps == 0) fq[1] = so_out;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const unsigned mine = TILE * ps + WPOS * x < TILE + f2_halo(c, a.PW) ? plane_off(c, 0, 0) : S2_OOB;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const unsigned o = (unsigned)__builtin_amdgcn_ds_bpermute((prow + 8 * u) * 4, (int)mine) + chunk16;
                    v[ps][4 * c + u] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, o, 0, 0);
                }
            }
        }
        // ---- the filter through LDS into operand registers: wf[s][ni] = wpk[32*ni + frow][16*s + 8*fk .. + 7]
#pragma unroll
        for (int u = 0; u < 18; ++u) {
            const int i = tid + 256 * u, row = i / 72, vv = i - row * 72;
            *(u32x4 *)(smem + row * S2_W_STRIDE + vv * 16) = wtmp[u];
        }
        lds_barrier();
        const unsigned char *wl = smem + frow * S2_W_STRIDE + fk * 16;
#pragma unroll
        for (int s = 0; s < 36; ++s)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) wf[s][ni] = *(const bf16x8 *)(wl + ni * 32 * S2_W_STRIDE + s * 32);
#pragma unroll
        for (int s = 0; s < F2_AGPR_STEPS; ++s)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) asm volatile("" : "+a"(wf[s][ni]));
        lds_barrier();                                           // everyone has read the filter: the rings may be written
#pragma unroll
        for (int ps = 0; ps < 2; ++ps)
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    // (rows past TILE + halo hold zeros here and are written again, with tile 1's rows, during tile 0)
                    const unsigned r = (unsigned)(TILE * ps + WPOS * x + prow + 8 * u);
                    lds_put<u32x4>(row_addr(c, r) + chunk16, 0, v[ps][4 * c + u]);
                }
        // the rows tile 1 needs beyond tile 0's (plane c: rows [TILE + halo_c, 2*TILE + halo_c)) are requested now and
        // go to the rings during tile 0; from then on the rows of tile p+2 are requested during tile p
        so1(1 < n ? Q0 + TILE + WPOS * x + (lane & 31) : 0x40000000);
        so2();
        so3();
        fq[2] = so_out;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const unsigned mine = plane_off_halo(c);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const unsigned o = (unsigned)__builtin_amdgcn_ds_bpermute((prow + 8 * u) * 4, (int)mine) + chunk16;
                st[4 * c + u] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, o, 0, 0);
            }
        }
    }

    // this lane's LDS addresses: fragment rows of the nine taps (tile 0), staging rows of the sixteen pieces (the rows
    // tile 1 adds), and its places in the wavefront's strip (rows 32x .. 32x+31 of plane (1,1), tile parity 0)
    unsigned ta[9], wa[16];
#pragma unroll
    for (int t = 0; t < 9; ++t)
        ta[t] = row_addr(f2_plane(t), (unsigned)(x * WPOS + frow + (f2_shift(t) >> 1) * a.PW + (f2_shift(t) & 1))) + (unsigned)fk * 16u;
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int u = 0; u < 4; ++u) wa[4 * c + u] = row_addr(c, (unsigned)(TILE + f2_halo(c, a.PW) + WPOS * x + prow + 8 * u)) + chunk16;
    const unsigned strip_w = row_addr(3, (unsigned)(WPOS * x + frow)) + (unsigned)fk * 8u;
    const unsigned strip_r = row_addr(3, (unsigned)(WPOS * x + prow)) + chunk16;     // + 8g rows = g * 4 row pairs
    unsigned mineI[4], offI[2];
    u32x4 sv[4];
    unsigned ooff[4];

    f32x16 acc[2];
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    lds_barrier();

    auto stats_dword = [&](unsigned w, int d) {
        const float lo = __builtin_bit_cast(float, w << 16), hi = __builtin_bit_cast(float, w & 0xFFFF0000u);
        ssum[2 * d] += lo;
        ssq[2 * d] += lo * lo;
        ssum[2 * d + 1] += hi;
        ssq[2 * d + 1] += hi * hi;
    };

    for (int p = 0; p < n; ++p) {
        // the strip of tile p-1 (read now) and of tile p (written at the end): the half of plane (1,1)'s ring that the
        // tile has consumed
        const unsigned tog_r = (unsigned)((p + 1) & 1) * ADV, tog_w = (unsigned)(p & 1) * ADV;
        bf16x8 af[DIST + 1];
        auto fetch = [&](auto pc) {
            constexpr int pair = decltype(pc)::value;
            af[pair % (DIST + 1)] = lds_get<bf16x8>(ta[pair >> 2], 2 * (pair & 3));
        };
        auto side = [&](auto sc) {
            constexpr F2Act act = f2_action(decltype(sc)::value);
            constexpr int k = act.kind, g = act.arg;
            // input rows of tile p+2: this lane computes the offsets of row WPOS*x + lane%32 of each plane
            if constexpr (k == F2_IA1) so1(p + 2 < n ? Q0 + TILE * (p + 2) + WPOS * x + (lane & 31) : 0x40000000);
            if constexpr (k == F2_IA2) so2();
            if constexpr (k == F2_IA3) so3();
            if constexpr (k == F2_IP) {
                mineI[g] = plane_off_halo(g);
                if constexpr (g == f2_piece_c(0)) offI[0] = (unsigned)__builtin_amdgcn_ds_bpermute((prow + 8 * f2_piece_u(0)) * 4, (int)mineI[g]);
            }
            // output vector g of tile p-1: strip -> registers, then to y
            if constexpr (k == F2_OR) {
                sv[g] = lds_get<u32x4>(strip_r + tog_r, g * (4 * F2_PAIR_BYTES / 16));
                ooff[g] = (unsigned)__builtin_amdgcn_ds_bpermute((prow + 8 * g) * 4, (int)fq[0]);
            }
            if constexpr (k == F2_OS) {
                __builtin_amdgcn_raw_buffer_store_b128(sv[g], out_rsrc, ooff[g] + chunk16, 0, 0);
                if constexpr (STATS) {                           // padding positions are neither stored nor counted
                    if (ooff[g] >= S2_OOB) sv[g] = u32x4{0u, 0u, 0u, 0u};
                }
            }
            if constexpr (k == F2_ST && STATS) {
                stats_dword(sv[g >> 1][2 * (g & 1)], 2 * (g & 1));
                stats_dword(sv[g >> 1][2 * (g & 1) + 1], 2 * (g & 1) + 1);
            }
            if constexpr (k == F2_TAPU) ta[g] = advance(ta[g], f2_plane(g));
            // input piece j = g: what was requested a tile ago goes to the ring, the same registers take the rows of
            // tile p+2; one slot later the ring address moves on and the next piece's offset is fetched from its lane
            if constexpr (k == F2_CLW) {
                constexpr int c = f2_piece_c(g), u = f2_piece_u(g);
                lds_put<u32x4>(wa[4 * c + u], 0, st[4 * c + u]);
                st[4 * c + u] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, offI[g & 1] + chunk16, 0, 0);
            }
            if constexpr (k == F2_CLA) {
                constexpr int c = f2_piece_c(g), u = f2_piece_u(g);
                wa[4 * c + u] = advance(wa[4 * c + u], c);
                if constexpr (g + 1 < 16)
                    offI[(g + 1) & 1] = (unsigned)__builtin_amdgcn_ds_bpermute((prow + 8 * f2_piece_u(g + 1)) * 4, (int)mineI[f2_piece_c(g + 1)]);
            }
        };
        static_for<0, DIST>([&](auto pc) { fetch(pc); });
        static_for<0, 2 * NPAIR>([&](auto ic) {
            constexpr int i = decltype(ic)::value, pair = i >> 1, ni = i & 1;
            if constexpr (ni == 0 && pair + DIST < NPAIR) fetch(std::integral_constant<int, pair + DIST>{});
            side(ic);
            __builtin_amdgcn_sched_barrier(0);
            acc[ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[pair][ni], af[pair % (DIST + 1)], pair == 0 ? zero16 : acc[ni], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        });
        // acc[ni][4g+j] is channel 32ni + 8g + 4fk + j of position frow: piece e = 4*ni + g converts four of them and
        // writes 8 bytes of the strip (row frow, 16-byte chunk e)
        static_for<0, 8>([&](auto ec) {
            constexpr int ni = decltype(ec)::value >> 2, g = decltype(ec)::value & 3;
            bf16x4 pk;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) pk[jj] = (bf16_t)acc[ni][g * 4 + jj];
            lds_put<bf16x4>(strip_w + tog_w, 2 * (ni * 4 + g), pk);
        });
        fq[0] = fq[1];
        fq[1] = fq[2];
        fq[2] = so_out;
        lds_barrier();
    }
    // the last tile's outputs
    const unsigned tog_r = (unsigned)((n + 1) & 1) * ADV;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const u32x4 v = lds_get<u32x4>(strip_r + tog_r, g * (4 * F2_PAIR_BYTES / 16));
        const unsigned o = (unsigned)__builtin_amdgcn_ds_bpermute((prow + 8 * g) * 4, (int)fq[0]);
        __builtin_amdgcn_raw_buffer_store_b128(v, out_rsrc, o + chunk16, 0, 0);
        if (STATS && o < S2_OOB) {
#pragma unroll
            for (int d = 0; d < 4; ++d) stats_dword(v[d], d);
        }
    }
    write_stats();
}

}  // namespace

// True if the launches described by a[0..count) are the four residue classes of the backward-data pass of a bf16 3x3
// stride-2 pad-1 64 -> 64 layer on even extents, in the order and with the tap order the kernel's schedule assumes.
bool fs64_dgrad_s2_applicable(int dtype, const IgemmArgs *a, int count)
{
    if (dtype != NSK_BF16 || count != 4 || hooks().no_fs) return false;
    static const int taps[4] = {1, 2, 2, 4};
    for (int c = 0; c < 4; ++c) {
        const IgemmArgs &g = a[c];
        if (g.Cs != 64 || g.Ngemm != 64 || g.Co != 64 || g.ntaps != taps[c] || g.accumulate || g.stats || g.zero_cell) return false;
        if (g.groups > 1 || g.osh != 2 || g.osw != 2 || g.oa != (c >> 1) || g.ob != (c & 1)) return false;
        if (g.mult_h != 1 || g.mult_w != 1 || g.add_h != 0 || g.add_w != 0) return false;
        if (g.Ho != 2 * g.Hs || g.Wo != 2 * g.Ws || g.Mi != g.Hs || g.Mj != g.Ws) return false;
        if (g.src != a[0].src || g.out != a[0].out || g.Nimg != a[0].Nimg || g.Hs != a[0].Hs || g.Ws != a[0].Ws) return false;
        for (int t = 0; t < g.ntaps; ++t)
            if (g.off_h[t] * 2 + g.off_w[t] != s2_shift(c, t) || g.off_h[t] < 0 || g.off_w[t] < 0) return false;
        if (((uintptr_t)g.src | (uintptr_t)g.wpk | (uintptr_t)g.out) & 15) return false;
    }
    const IgemmArgs &g = a[0];
    if (2 * S2_TILE + g.Ws + 2 > S2_RING_MAX) return false;
    const long long pi = (long long)(g.Hs + 1) * (g.Ws + 1), total = pi * g.Nimg;
    if (total >= (1LL << 30) || total * pi >= (1LL << 40)) return false;   // exactness of the reciprocal division
    const unsigned long long out_bytes = (unsigned long long)g.Nimg * g.Ho * g.Wo * 64 * 2;
    if ((unsigned long long)g.src_bytes >= S2_OOB || out_bytes + 4096 >= S2_OOB) return false;
    // worth it only when the tiles fill a good part of the chip
    return total >= 64 * S2_TILE;
}

// True for the forward pass of a bf16 3x3 stride-2 pad-1 64 -> 64 layer on even extents, taps in (r, s) order.
bool fs64_fwd_s2_applicable(int dtype, const IgemmArgs &g)
{
    if (dtype != NSK_BF16 || hooks().no_fs) return false;
    if (g.Cs != 64 || g.Ngemm != 64 || g.Co != 64 || g.ntaps != 9 || g.Ktot != 576 || g.accumulate || g.zero_cell || g.groups > 1 || g.act) return false;
    if (g.mult_h != 2 || g.mult_w != 2 || g.add_h != -1 || g.add_w != -1 || g.osh != 1 || g.osw != 1 || g.oa != 0 || g.ob != 0) return false;
    if (g.Hs % 2 != 0 || g.Ws % 2 != 0 || g.Mi != g.Hs / 2 || g.Mj != g.Ws / 2 || g.Ho != g.Mi || g.Wo != g.Mj) return false;
    for (int t = 0; t < 9; ++t)
        if (g.off_h[t] != t / 3 || g.off_w[t] != t % 3) return false;
    if (((uintptr_t)g.src | (uintptr_t)g.wpk | (uintptr_t)g.out) & 15) return false;
    const int PW = g.Mj + 1;
    if (PW > F2_MAX_PW) return false;
    const long long pi = (long long)(g.Mi + 1) * PW, total = pi * g.Nimg;
    if (total >= (1LL << 30) || total * pi >= (1LL << 40) || pi * PW >= (1LL << 40)) return false;   // exactness of the reciprocal divisions
    if ((unsigned long long)g.src_bytes + 4096 >= S2_OOB) return false;
    // worth it only when the tiles fill a good part of the chip
    return total >= 128LL * F2_TILE;
}

static int f2_grid(const IgemmArgs &g, int want)
{
    const int tiles = ceil_div((g.Mi + 1) * (g.Mj + 1) * g.Nimg, F2_TILE);
    return tiles < want ? tiles : want;
}

// Rows of partial sums the forward launch writes: one per wavefront
int fs64_fwd_s2_stats_rows(const IgemmArgs &g) { return f2_grid(g, F2_STATS_GRID) * 4; }

int launch_fs64_fwd_s2(const IgemmArgs &g, hipStream_t stream)
{
    F2Args a{};
    a.src = g.src; a.wpk = g.wpk; a.out = g.out;
    a.stats = g.stats; a.stats_rows = g.stats_rows;
    a.N = g.Nimg; a.H = g.Hs; a.W = g.Ws; a.P = g.Mi; a.Q = g.Mj;
    a.PW = a.Q + 1; a.PR = a.P + 1; a.PI = a.PR * a.PW;
    a.total_pos = a.PI * a.N;
    a.tiles = ceil_div(a.total_pos, F2_TILE);
    a.img_bytes = (unsigned)(a.H * a.W * 128);
    a.row2_bytes = (unsigned)(2 * a.W * 128);
    a.magic_pi = ((1ULL << 40) + a.PI - 1) / a.PI;
    a.magic_pw = ((1ULL << 40) + a.PW - 1) / a.PW;
    a.src_bytes = g.src_bytes;
    a.out_bytes = (unsigned)((size_t)g.Nimg * g.Ho * g.Wo * 64 * 2);
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return NSK_ERR_HIP;
        cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    }
    const int grid = f2_grid(g, g.stats ? F2_STATS_GRID : cus);
    if (g.stats && g.stats_rows != grid * 4) return NSK_ERR_BAD_DESC;   // the planner and the launch disagree
    const int smem = f2_lds_bytes(a.PW);
    static bool attr_set = false;
    if (!attr_set) {
        const int smem_max = f2_lds_bytes(F2_MAX_PW);
        hipError_t e = hipFuncSetAttribute((const void *)conv_fs64_fwd_s2_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_max);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)conv_fs64_fwd_s2_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_max);
        if (e != hipSuccess) {
            set_last_hip_error(e);
            return NSK_ERR_HIP;
        }
        attr_set = true;
    }
    if (g.stats)
        hipLaunchKernelGGL(conv_fs64_fwd_s2_kernel<true>, dim3(grid), dim3(256), smem, stream, a);
    else
        hipLaunchKernelGGL(conv_fs64_fwd_s2_kernel<false>, dim3(grid), dim3(256), smem, stream, a);
    return check_launch();
}

int launch_fs64_dgrad_s2(const IgemmArgs *g, int count, hipStream_t stream)
{
    if (count != 4) return NSK_ERR_BAD_DESC;
    S2Args a{};
    a.src = g[0].src; a.out = g[0].out;
    for (int c = 0; c < 4; ++c) {
        a.wpk[c] = g[c].wpk;
        a.oshift[c] = (unsigned)(((c >> 1) * g[0].Wo + (c & 1)) * 64 * 2);
    }
    a.N = g[0].Nimg; a.Hs = g[0].Hs; a.Ws = g[0].Ws;
    a.PW = a.Ws + 1; a.PI = (a.Hs + 1) * a.PW;
    a.total_pos = a.PI * a.N;
    a.tiles = ceil_div(a.total_pos, S2_TILE);
    a.halo = a.PW + 1;
    a.magic_pi = ((1ULL << 40) + a.PI - 1) / a.PI;
    a.magic_pw = ((1ULL << 40) + a.PW - 1) / a.PW;
    a.src_bytes = g[0].src_bytes;
    a.out_bytes = (unsigned)((size_t)g[0].Nimg * g[0].Ho * g[0].Wo * 64 * 2);
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return NSK_ERR_HIP;
        cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    }
    const int grid = a.tiles < cus ? a.tiles : cus;
    const int smem = S2_RING_MAX * S2_SLOT + 4 * 2 * S2_WPOS * S2_SLOT;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)conv_fs64_dgrad_s2_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) {
            set_last_hip_error(e);
            return NSK_ERR_HIP;
        }
        attr_set = true;
    }
    hipLaunchKernelGGL(conv_fs64_dgrad_s2_kernel, dim3(grid), dim3(256), smem, stream, a);
    return check_launch();
}

}  // namespace nsk

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

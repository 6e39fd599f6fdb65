// 3x3, stride 1, 64 -> 64 channel fp32 convolution (forward, and backward-data through the packed
// transposed filter): the fp32 sibling of conv_halo64.hip, for the small-image residual blocks the
// paper trains in fp32 (section "Experiments and Discussion").
//
// Same scheme: zero-padded coordinates (a tap is one constant shift, image borders need no special
// case), persistent blocks that walk over tiles, the input tile staged ONCE with its halo and read at
// shifted rows by all nine taps, the next tile prefetched into registers while the MFMAs of the current
// one run, and an epilogue that transposes through LDS so that every lane stores 16 contiguous bytes.
//
// Tiles are ROW ALIGNED here: the kernel takes images that are 32 pixels wide (the small-image
// workloads), a 32-row MFMA fragment is exactly one image row, a tile is 8 rows of one image, and the
// staged region is those rows plus one above and below, each with its two padding columns.  No
// matrix work is spent on padding positions, and N*H/8 tiles divide evenly over the CUs for the
// configured batch sizes (an fp32 tile is long, so a ragged last round of tiles would cost 10-25%).
//
// What differs from bf16: the fp32 filter (144 KB) does not fit in LDS beside the input tile, so it is
// streamed one tap (64 x 64 floats) at a time through two LDS buffers: the tap after the current one
// is fetched from L2 while the current one is multiplied (an fp32 32x32x2 MFMA lasts 64 clocks, so a
// tap is 8192 clocks of matrix work per wavefront and the 16 KB fetch hides easily).  One barrier per
// tap.  The epilogue staging reuses the input tile's LDS after the last tap.
//
// Lane (row, half) of a fragment holds reduction index 4*half + t of each group of 8 channels for both
// operands (t = 0..3 over four consecutive MFMAs), which makes every fragment one 16-byte LDS read.
#include "nsk_internal.h"

namespace nsk {
namespace {

constexpr int F_W = 32;            // image width this kernel takes
constexpr int F_MAX_IN = 352;      // 10 rows of W+2 = 340 staged positions, rounded up to a multiple of 16
constexpr int F_ROW = 272;         // bytes per staged position / filter row (64 floats + 16 pad)
constexpr int F_PASSES = F_MAX_IN / 16;   // 16 lanes of 16 bytes per position, 16 positions per pass
constexpr unsigned F_OOB = 0xF0000000u;
constexpr int F_WBUF = 64 * F_ROW;  // one tap of the filter

struct HaloF32Args {
    const void *src, *wpk;
    void *out;
    int N, H, W, PW, PI;
    int total_pos, tiles, tiles_per_img;
    unsigned long long magic_pi, magic_pw;
    unsigned src_bytes, wpk_bytes;
    int tapoff[9];
    float *stats;      // forward only: per-channel partial sums of the stored output, or nullptr
    int stats_rows;    // 4 rows per block (one per wavefront)
    const float *act;  // nullptr, or [2][64]: the input is relu(act[c]*src + act[64+c]), applied while the tile is staged
};

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <bool ACCUM, bool ACT = false>
__global__ __launch_bounds__(256) void conv_halo64_f32_kernel(const HaloF32Args a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char *in_lds = smem;                                   // F_MAX_IN * 272 (also epilogue staging)
    unsigned char *w_lds = smem + F_MAX_IN * F_ROW;                 // 2 taps
    unsigned *out_tab = (unsigned *)(w_lds + 2 * F_WBUF);           // 256
    unsigned *in_tab = out_tab + 256;                               // F_MAX_IN

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int frow = lane & 31, fk = lane >> 5;
    const __amdgpu_buffer_rsrc_t src_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.src, 0, a.src_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t out_rsrc = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, a.src_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.wpk, 0, a.wpk_bytes, 0x00020000);
    const int n_in = 10 * a.PW;
    const int chunk = tid & 15, prow = tid >> 4;

    auto src_offset = [&](int q) -> unsigned {
        const bool inside = (unsigned)q < (unsigned)a.total_pos;
        const unsigned qq = inside ? (unsigned)q : 0u;
        const unsigned img = (unsigned)(((unsigned long long)qq * a.magic_pi) >> 40);
        const unsigned rem = qq - img * (unsigned)a.PI;
        const unsigned hp = (unsigned)(((unsigned long long)rem * a.magic_pw) >> 40);
        const unsigned wp = rem - hp * (unsigned)a.PW;
        const bool ok = inside & (hp - 1u < (unsigned)a.H) & (wp - 1u < (unsigned)a.W);
        const unsigned off = (((img * a.H + (hp - 1u)) * a.W + (wp - 1u)) * 64u) * 4u;
        return ok ? off : F_OOB;
    };
    // first staged position of a tile: padded row h0 of its image is the real row above the tile
    auto tile_q0 = [&](int tile) { return (tile / a.tiles_per_img) * a.PI + (tile % a.tiles_per_img) * 8 * a.PW; };
    auto fill_in_tab = [&](int tile, bool live) {   // !live: a table of out-of-range offsets (loads that fetch nothing)
        const int q0 = live ? tile_q0(tile) : 0;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int p = tid + 256 * u;
            if (p < F_MAX_IN) in_tab[p] = live && p < n_in ? src_offset(q0 + p) : F_OOB;
        }
    };
    u32x4 stage[F_PASSES];
    // ACT: a thread always stages the same four channels (4*chunk ..): their coefficients live in registers, and one
    // bit per pass remembers whether the position was real (padding must stay zero, not relu(shift))
    float asc[4] = {0.f, 0.f, 0.f, 0.f}, ash[4] = {0.f, 0.f, 0.f, 0.f};
    if (ACT) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            asc[e] = a.act[chunk * 4 + e];
            ash[e] = a.act[64 + chunk * 4 + e];
        }
    }
    unsigned real_bits = 0;
    auto prefetch_tile = [&]() {   // reads the table that fill_in_tab wrote before the last barrier
        real_bits = 0;
#pragma unroll
        for (int u = 0; u < F_PASSES; ++u) {
            const unsigned off = in_tab[u * 16 + prow];
            stage[u] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, off == F_OOB ? F_OOB : off + chunk * 16, 0, 0);
            if (ACT) real_bits |= (off != F_OOB ? 1u : 0u) << u;
        }
    };
    // filter tap t: rows n = 0..63, 64 floats each at wpk[n][t][0..63]; 4 vectors per thread
    u32x4 wreg[4];
    auto load_tap = [&](int t) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = tid + 256 * u, n = idx >> 4, v = idx & 15;
            wreg[u] = __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, (unsigned)(((n * 9 + t) * 64 + v * 4) * 4), 0, 0);
        }
    };
    auto store_tap = [&](int buf) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = tid + 256 * u, n = idx >> 4, v = idx & 15;
            *(u32x4 *)(w_lds + buf * F_WBUF + n * F_ROW + v * 16) = wreg[u];
        }
    };

    // statistics epilogue (forward): a lane reads back the same 4 channels of every staged row and adds them up over
    // all the positions it stores during the life of the block; each wavefront leaves one row of partial sums
    float ssum[4] = {0.f, 0.f, 0.f, 0.f}, ssq[4] = {0.f, 0.f, 0.f, 0.f};
    int tile = blockIdx.x;
    int wb = 0;   // LDS buffer holding the tap about to be multiplied
    if (tile < a.tiles) {
        fill_in_tab(tile, true);
        load_tap(0);
        store_tap(0);
        __syncthreads();
        prefetch_tile();
    }
    // wavefront w owns tile rows 2w and 2w+1; staged index of pixel (row r, column c) is (r+1)*PW + c+1
    const unsigned a_base0 = (unsigned)((((2 * wave + 1) * a.PW) + 1 + frow) * F_ROW + fk * 16);
    const unsigned a_row = (unsigned)(a.PW * F_ROW);
    const unsigned b_base0 = (unsigned)(frow * F_ROW + fk * 16);

    for (; tile < a.tiles; tile += gridDim.x) {
#pragma unroll
        for (int u = 0; u < F_PASSES; ++u) {
            const int p = u * 16 + prow;
            if (ACT) {
                f32x4 v = __builtin_bit_cast(f32x4, stage[u]);
                const bool real = (real_bits >> u) & 1u;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float z = v[e] * asc[e] + ash[e];   // the expression of the batch-norm apply pass
                    v[e] = real && z > 0.f ? z : 0.f;
                }
                stage[u] = __builtin_bit_cast(u32x4, v);
            }
            if (p < n_in) *(u32x4 *)(in_lds + p * F_ROW + chunk * 16) = stage[u];
        }
        {   // tile pixel tid = (row tid/32, column tid%32): always a real pixel
            const int img = tile / a.tiles_per_img, h0 = (tile % a.tiles_per_img) * 8;
            out_tab[tid] = (unsigned)((((img * a.H + h0) * F_W) + tid) * 64 * 4);
        }
        const int next = tile + (int)gridDim.x;
        const bool have_next = next < a.tiles;
        fill_in_tab(next, have_next);
        __syncthreads();

        // filter rows are the MFMA "A" operand, positions the "B" operand: acc[ni][mi][4g+j] is channel
        // 32*ni + 8*g + 4*(lane/32) + j of position 32*mi + lane%32
        f32x16 acc[2][2];
        if (ACCUM) {
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) {
                const unsigned off = out_tab[wave * 64 + mi * 32 + frow];
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const unsigned o = off == F_OOB ? F_OOB : off + (unsigned)((ni * 32 + g * 8 + fk * 4) * 4);
                        const f32x4 old = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(out_rsrc, o, 0, 0));
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj) acc[ni][mi][g * 4 + jj] = old[jj];
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

        // One tap: the tap after it (tap 0 of the next tile after the last) goes global -> registers before the MFMAs and
        // registers -> the other LDS buffer after them; the barrier orders LDS only, so loads stay in flight across it.
        auto multiply_tap = [&](int t) {
            const unsigned char *pa = in_lds + a_base0 + a.tapoff[t] * F_ROW;
            const unsigned char *pb = w_lds + wb * F_WBUF + b_base0;
            f32x4 xf[2][2], wf[2][2];
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) xf[0][mi] = *(const f32x4 *)(pa + mi * a_row);
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) wf[0][ni] = *(const f32x4 *)(pb + ni * 32 * F_ROW);
#pragma unroll
            for (int g = 0; g < 8; ++g) {
                if (g + 1 < 8) {
#pragma unroll
                    for (int mi = 0; mi < 2; ++mi) xf[(g + 1) & 1][mi] = *(const f32x4 *)(pa + mi * a_row + (g + 1) * 32);
#pragma unroll
                    for (int ni = 0; ni < 2; ++ni) wf[(g + 1) & 1][ni] = *(const f32x4 *)(pb + ni * 32 * F_ROW + (g + 1) * 32);
                }
#pragma unroll
                for (int tt = 0; tt < 4; ++tt)
#pragma unroll
                    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                        for (int ni = 0; ni < 2; ++ni)
                            acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x2f32(wf[g & 1][ni][tt], xf[g & 1][mi][tt], acc[ni][mi], 0, 0, 0);
            }
            store_tap(wb ^ 1);
            wb ^= 1;
            lds_barrier();
        };
        // Tap 0 apart from the loop: its filter successor is requested BEFORE the next tile.  A wavefront's loads return
        // in order and every block asks for its next tile at the same moment, so whatever is requested behind that burst
        // of HBM loads arrives late; this way nothing is needed from behind it for two taps.  (Without a next tile the
        // table holds out-of-range offsets and the same loads fetch nothing: no branch around them, so the compiler's
        // wait counts stay exact.)
        load_tap(1);
        prefetch_tile();
        multiply_tap(0);
#pragma unroll 1
        for (int t = 1; t < 9; ++t) {
            load_tap(t == 8 ? 0 : t + 1);
            multiply_tap(t);
        }
        __syncthreads();   // also: every wavefront is done with the input tile, it becomes the epilogue staging area

        // Epilogue through this wavefront's strip of the (now idle) input tile: 32 positions x 272 B
        unsigned char *my_st = in_lds + wave * (32 * F_ROW);
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    f32x4 pk;
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) pk[jj] = acc[ni][mi][g * 4 + jj];
                    *(f32x4 *)(my_st + frow * F_ROW + (ni * 32 + g * 8 + fk * 4) * 4) = pk;
                }
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
                const int idx = lane + 64 * jj, pos = idx >> 4, ck = idx & 15;
                const u32x4 v = *(const u32x4 *)(my_st + pos * F_ROW + ck * 16);
                const unsigned off = out_tab[wave * 64 + mi * 32 + pos];
                __builtin_amdgcn_raw_buffer_store_b128(v, out_rsrc, off == F_OOB ? F_OOB : off + (unsigned)(ck * 16), 0, 0);
                if (!ACCUM && a.stats && off != F_OOB) {
                    const f32x4 vf = __builtin_bit_cast(f32x4, v);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        ssum[e] += vf[e];
                        ssq[e] += vf[e] * vf[e];
                    }
                }
            }
        }
        __syncthreads();
    }
    if (!ACCUM && a.stats) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int o = 16; o < 64; o <<= 1) {
                ssum[e] += __shfl_xor(ssum[e], o, 64);
                ssq[e] += __shfl_xor(ssq[e], o, 64);
            }
        if (lane < 16) {
            float *r0 = a.stats + (size_t)(blockIdx.x * 4 + wave) * 64 + lane * 4;
            float *r1 = r0 + (size_t)a.stats_rows * 64;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                r0[e] = ssum[e];
                r1[e] = ssq[e];
            }
        }
    }
}

constexpr int kSmemF32 = F_MAX_IN * F_ROW + 2 * F_WBUF + 256 * 4 + F_MAX_IN * 4;

}  // namespace

bool halo64_f32_applicable(int dtype, const IgemmArgs &a)
{
    if (dtype != NSK_F32 || a.Cs != 64 || a.Ngemm != 64 || a.ntaps != 9 || a.Co != 64) return false;
    if (a.mult_h != 1 || a.mult_w != 1 || a.osh != 1 || a.osw != 1 || a.oa != 0 || a.ob != 0) return false;
    if (a.Hs != a.Ho || a.Ws != a.Wo || a.Mi != a.Ho || a.Mj != a.Wo) return false;
    if (a.Ws != F_W || a.Hs % 8 != 0) return false;
    for (int t = 0; t < 9; ++t) {
        const int eh = a.add_h + a.off_h[t], ew = a.add_w + a.off_w[t];
        if (eh < -1 || eh > 1 || ew < -1 || ew > 1) return false;
    }
    const long long pi = (long long)(a.Hs + 2) * (a.Ws + 2), total = pi * a.Nimg;
    if (total >= (1LL << 30) || total * pi >= (1LL << 40)) return false;
    if ((unsigned long long)a.src_bytes >= F_OOB) return false;
    if (((uintptr_t)a.src | (uintptr_t)a.wpk | (uintptr_t)a.out) & 15) return false;
    return true;
}

namespace {
constexpr int kStatsGridF32 = 256;   // block count when statistics are requested (independent of the device)
}

// Rows of partial sums the forward launch writes (4 per block).
int halo64_f32_stats_rows(const IgemmArgs &g)
{
    if (g.accumulate) return 0;
    const int tiles = g.Nimg * (g.Hs / 8);
    return (tiles < kStatsGridF32 ? tiles : kStatsGridF32) * 4;
}

int launch_halo64_f32(const IgemmArgs &g, hipStream_t stream)
{
    HaloF32Args a{};
    a.src = g.src; a.wpk = g.wpk; a.out = g.out;
    a.N = g.Nimg; a.H = g.Hs; a.W = g.Ws;
    a.PW = g.Ws + 2; a.PI = (g.Hs + 2) * a.PW;
    a.total_pos = a.PI * g.Nimg;
    a.tiles_per_img = g.Hs / 8;
    a.tiles = g.Nimg * a.tiles_per_img;
    a.magic_pi = ((1ULL << 40) + a.PI - 1) / a.PI;
    a.magic_pw = ((1ULL << 40) + a.PW - 1) / a.PW;
    a.src_bytes = g.src_bytes;
    a.wpk_bytes = g.wpk_bytes;
    for (int t = 0; t < 9; ++t) a.tapoff[t] = (g.add_h + g.off_h[t]) * a.PW + (g.add_w + g.off_w[t]);
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return NSK_ERR_HIP;
        cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    }
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)conv_halo64_f32_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, kSmemF32);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)conv_halo64_f32_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, kSmemF32);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)conv_halo64_f32_kernel<false, true>, hipFuncAttributeMaxDynamicSharedMemorySize, kSmemF32);
        if (e != hipSuccess) {
            set_last_hip_error(e);
            return NSK_ERR_HIP;
        }
        attr_set = true;
    }
    const int want = g.stats ? kStatsGridF32 : cus;
    const int grid = a.tiles < want ? a.tiles : want;
    if (g.stats && g.stats_rows != grid * 4) return NSK_ERR_BAD_DESC;   // the planner and the launch disagree
    a.stats = g.stats;
    a.stats_rows = g.stats_rows;
    a.act = g.act;
    if (g.act && g.accumulate) return NSK_ERR_BAD_DESC;   // the fused load belongs to the forward pass
    if (g.act)
        hipLaunchKernelGGL((conv_halo64_f32_kernel<false, true>), dim3(grid), dim3(256), kSmemF32, stream, a);
    else if (g.accumulate)
        hipLaunchKernelGGL(conv_halo64_f32_kernel<true>, dim3(grid), dim3(256), kSmemF32, stream, a);
    else
        hipLaunchKernelGGL(conv_halo64_f32_kernel<false>, dim3(grid), dim3(256), kSmemF32, stream, a);
    return check_launch();
}

}  // namespace nsk

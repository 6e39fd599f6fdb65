// Forward and backward-data of the 7x7 stride-2 image stem on its space-to-depth copy (see conv_stem.hip:
// a 4x4 stride-1 filter over 16 channels; the ResNet recipe of the paper's section "Experiments and
// Discussion" starts with this layer), bf16, 64 output channels.
//
// Both passes are bound by memory and LDS traffic, not by the matrix units (the forward pass writes 128 bytes
// per position for 32 bytes read; the backward pass produces only 16 numbers per position), so what matters is
// that every byte crosses HBM once and every position is staged in LDS once for all sixteen taps.  Same scheme as
// the 3x3 64->64 kernel: flat zero-padded coordinates (the coarse image is padded by 2 rows/columns before and 1
// after for the forward pass, 1 before and 2 after for the backward pass; a tap is a constant shift and padding
// positions load zeros through out-of-range buffer offsets), tiles of 256 consecutive positions staged with their
// halo, the whole filter resident in LDS, persistent blocks over contiguous runs of tiles, the next tile's loads
// issued into registers behind the MFMAs of the current one.
//
//   forward        y[pos][k]   = sum_{t,c}  x2[pos + shift_t][c] * w2[k][t][c]        (16 taps x 16 channels)
//   backward-data  dx2[pos][e] = sum_{t,k}  dy[pos - shift_t][k] * w2[k][t][e]        (16 taps x 64 channels)
// The backward pass has 16 outputs per position; they occupy half of a 32-row MFMA tile (the other rows of the
// filter tile are zero).
#include <stdlib.h>

#include "nsk_internal.h"

namespace nsk {
namespace {

constexpr int SH_T = 256;              // positions per tile
constexpr int SH_MAX_IN = 608;         // staged positions incl. halo: 256 + 3*(PW+1) <= 608  ->  PW <= 116
constexpr unsigned SH_OOB = 0xF0000000u;

struct StemHaloArgs {
    const void *src, *wpk;
    void *out;
    int H, W;                          // coarse image size (input and output grids are the same)
    int PW, PI, padlo;                 // padded width, padded image size, padding before
    int total_pos, tiles, halo_lo, halo_hi;
    unsigned long long magic_pi, magic_pw;   // ceil(2^40 / d)
    unsigned src_bytes, out_bytes;
    int tapoff[16];                    // shift of each tap in flat padded positions
    float *stats;                      // forward only: per-channel partial sums of the stored output, or nullptr
    int stats_rows;                    // 4 rows per block (one per wavefront)
};

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// CPP: 16-byte chunks per input position (2: forward, 16 channels; 8: backward-data, 64 channels)
// NT:  32-row tiles of filter rows (2: forward, 64 output channels; 1: backward-data, 16 of 32 rows used)
// OC:  output channels stored per position (64 / 16)
template <int CPP, int NT, int OC>
__global__ __launch_bounds__(256) void stem_halo_kernel(const StemHaloArgs a)
{
    constexpr int KC = CPP / 2;                    // 16-channel MFMA steps per tap
    constexpr int IN_ROW = CPP * 16 + 16;          // LDS bytes per staged position (conflict-free 16-byte reads)
    constexpr int FW_ROW = 16 * KC * 32 + 16;      // LDS bytes per filter row (16 taps x KC x 16 channels)
    constexpr int F_ROWS = NT * 32;
    constexpr int F_REAL = OC < F_ROWS ? OC : F_ROWS;   // filter rows that exist in memory
    constexpr int PPP = 256 / CPP;                 // positions staged per pass of the 256 threads
    constexpr int PASSES = (SH_MAX_IN + PPP - 1) / PPP;
    constexpr int STEPS = 16 * KC;
    constexpr int OUT_B = OC * 2;                  // bytes stored per position
    constexpr int O_CPP = OUT_B / 16;              // 16-byte chunks per output position
    constexpr int ST_ROW = OUT_B + 16;             // epilogue staging row
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char *in_lds = smem;                                   // SH_MAX_IN * IN_ROW (the epilogue strips alias it)
    unsigned char *w_lds = smem + SH_MAX_IN * IN_ROW;               // F_ROWS * FW_ROW
    unsigned *out_tab = (unsigned *)(w_lds + F_ROWS * FW_ROW);      // 256 pixel indices of the tile's outputs
    unsigned *in_tab = out_tab + 256;                               // SH_MAX_IN pixel indices of the next tile's inputs

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int frow = lane & 31, fk = lane >> 5;
    const __amdgpu_buffer_rsrc_t src_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.src, 0, a.src_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t out_rsrc = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, a.out_bytes, 0x00020000);

    // filter -> LDS once per block; rows beyond the real ones are zero
    {
        constexpr int VPR = 16 * KC * 2;           // 16-byte vectors per filter row
        const u32x4 *w = (const u32x4 *)a.wpk;
        for (int i = tid; i < F_ROWS * VPR; i += 256) {
            const int row = i / VPR, v = i - row * VPR;
            u32x4 val = {0u, 0u, 0u, 0u};
            if (row < F_REAL) val = w[row * VPR + v];
            *(u32x4 *)(w_lds + row * FW_ROW + v * 16) = val;
        }
    }

    // pixel index (image-major, row-major) of padded position q, or out of range
    auto pixel = [&](int q) -> unsigned {
        const bool inside = (unsigned)q < (unsigned)a.total_pos;
        const unsigned qq = inside ? (unsigned)q : 0u;
        const unsigned img = (unsigned)(((unsigned long long)qq * a.magic_pi) >> 40);
        const unsigned rem = qq - img * (unsigned)a.PI;
        const unsigned hp = (unsigned)(((unsigned long long)rem * a.magic_pw) >> 40);
        const unsigned wp = rem - hp * (unsigned)a.PW;
        const unsigned h = hp - (unsigned)a.padlo, w = wp - (unsigned)a.padlo;
        const bool ok = inside & (h < (unsigned)a.H) & (w < (unsigned)a.W);
        return ok ? (img * (unsigned)a.H + h) * (unsigned)a.W + w : SH_OOB;
    };

    const int n_in = SH_T + a.halo_lo + a.halo_hi;
    const int chunk = tid % CPP, prow = tid / CPP;
    u32x4 stage[PASSES];
    // in_tab[p] = pixel index of staged position p of the tile to be loaded next: computed by (up to) three
    // positions per thread, so the CPP lanes that share a position do not repeat the index arithmetic
    auto fill_in_tab = [&](int tile, bool live) {
#pragma unroll
        for (int u = 0; u < (SH_MAX_IN + 255) / 256; ++u) {
            const int p = tid + 256 * u;
            if (p < SH_MAX_IN) in_tab[p] = (live && p < n_in) ? pixel(tile * SH_T - a.halo_lo + p) : SH_OOB;
        }
    };
    // loads of one tile's staged positions: thread (prow, chunk) takes positions prow + PPP*u
    auto issue_tile = [&]() {
        unsigned off[PASSES];
#pragma unroll
        for (int u = 0; u < PASSES; ++u) {
            const int p = prow + PPP * u;
            const unsigned px = p < SH_MAX_IN ? in_tab[p] : SH_OOB;
            off[u] = px == SH_OOB ? SH_OOB : px * (unsigned)(CPP * 16) + (unsigned)(chunk * 16);
        }
#pragma unroll
        for (int u = 0; u < PASSES; ++u) stage[u] = __builtin_amdgcn_raw_buffer_load_b128(src_rsrc, off[u], 0, 0);
    };

    // Statistics epilogue (forward): a lane reads back the same 8 channels of every staged row; it adds them up over
    // all the positions it stores during the life of the block, and each wavefront leaves one row of partial sums.
    float ssum[8], ssq[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) ssum[e] = ssq[e] = 0.f;
    auto write_stats = [&]() {
        if (OC != 64 || !a.stats) return;
#pragma unroll
        for (int e = 0; e < 8; ++e)
#pragma unroll
            for (int o = 8; o < 64; o <<= 1) {
                ssum[e] += __shfl_xor(ssum[e], o, 64);
                ssq[e] += __shfl_xor(ssq[e], o, 64);
            }
        if (lane < 8) {
            float *r0 = a.stats + (size_t)(blockIdx.x * 4 + wave) * 64 + lane * 8;
            float *r1 = r0 + (size_t)a.stats_rows * 64;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                r0[e] = ssum[e];
                r1[e] = ssq[e];
            }
        }
    };
    const int tiles_per_block = (a.tiles + (int)gridDim.x - 1) / (int)gridDim.x;
    const int t_begin = blockIdx.x * tiles_per_block;
    const int t_end = min(a.tiles, t_begin + tiles_per_block);
    if (t_begin >= t_end) {   // uniform for the block
        write_stats();        // zeros: every row of the buffer is written
        return;
    }
    fill_in_tab(t_begin, true);
    __syncthreads();                // in_tab and the filter
    issue_tile();

    // fragment addressing: filter rows are the MFMA "A" operand, positions the "B" operand, so a lane holds 4
    // consecutive output channels of one position: acc[ni][mi][4g+j] = channel 32ni + 8g + 4fk + j of position 32mi + frow
    const unsigned a_base0 = (unsigned)((wave * 64 + frow + a.halo_lo) * IN_ROW + fk * 16);
    const unsigned b_base0 = (unsigned)(frow * FW_ROW + fk * 16);

    for (int tile = t_begin; tile < t_end; ++tile) {
        // staged registers -> LDS (the barrier at the end of the previous tile freed the buffer)
#pragma unroll
        for (int u = 0; u < PASSES; ++u) {
            const int p = prow + PPP * u;
            if (p < n_in) *(u32x4 *)(in_lds + p * IN_ROW + chunk * 16) = stage[u];
        }
        out_tab[tid] = pixel(tile * SH_T + tid);
        fill_in_tab(tile + 1, tile + 1 < t_end);   // the reads of the previous in_tab completed before its loads were issued
        lds_barrier();
        issue_tile();                              // lands in registers behind the MFMAs below

        unsigned ta[16];
#pragma unroll
        for (int t = 0; t < 16; ++t) ta[t] = a_base0 + (unsigned)(a.tapoff[t] * IN_ROW);
        f32x16 acc[NT][2];
#pragma unroll
        for (int ni = 0; ni < NT; ++ni)
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[ni][mi][v] = 0.f;
        bf16x8 af[3][2], bfr[3][NT];
        auto fetch = [&](int step, int set) {
            const int t = step / KC, kc = step % KC;
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) af[set][mi] = *(const bf16x8 *)(in_lds + ta[t] + mi * 32 * IN_ROW + kc * 32);
#pragma unroll
            for (int ni = 0; ni < NT; ++ni)
                bfr[set][ni] = *(const bf16x8 *)(w_lds + b_base0 + ni * 32 * FW_ROW + (t * KC + kc) * 32);
        };
        fetch(0, 0);
        fetch(1, 1);
#pragma unroll
        for (int step = 0; step < STEPS; ++step) {
            if (step + 2 < STEPS) fetch(step + 2, (step + 2) % 3);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int ni = 0; ni < NT; ++ni)
                    acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[step % 3][ni], af[step % 3][mi], acc[ni][mi], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        lds_barrier();   // every wavefront is done with the staged tile: its memory becomes the epilogue strips

        // Epilogue: round to bf16, transpose through this wavefront's strip, store 16 contiguous bytes per lane.
        unsigned char *my_st = in_lds + wave * (32 * ST_ROW);
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
#pragma unroll
            for (int ni = 0; ni < NT; ++ni)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int ch = ni * 32 + g * 8 + fk * 4;
                    if (ch < OC) {
                        bf16x4 pk;
#pragma unroll
                        for (int j = 0; j < 4; ++j) pk[j] = (bf16_t)acc[ni][mi][g * 4 + j];
                        *(bf16x4 *)(my_st + frow * ST_ROW + ch * 2) = pk;
                    }
                }
#pragma unroll
            for (int jj = 0; jj < (32 * O_CPP + 63) / 64; ++jj) {
                const int idx = lane + 64 * jj, pos = idx / O_CPP, ck = idx % O_CPP;
                if (pos < 32) {
                    const u32x4 v = *(const u32x4 *)(my_st + pos * ST_ROW + ck * 16);
                    const unsigned px = out_tab[wave * 64 + mi * 32 + pos];
                    const unsigned o = px == SH_OOB ? SH_OOB : px * (unsigned)OUT_B + (unsigned)(ck * 16);
                    __builtin_amdgcn_raw_buffer_store_b128(v, out_rsrc, o, 0, 0);
                    if (OC == 64 && a.stats && px != SH_OOB) {
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
        }
        lds_barrier();   // strips and out_tab are free again
    }
    write_stats();
}

template <int CPP, int NT, int OC> constexpr int stem_halo_smem()
{
    return SH_MAX_IN * (CPP * 16 + 16) + NT * 32 * (16 * (CPP / 2) * 32 + 16) + 256 * 4 + SH_MAX_IN * 4;
}

}  // namespace

// True if the 4x4-tap problem on the H x W coarse grid fits the kernels (7x7 stem, 64 output channels).
bool stem_halo_applicable(int dtype, int U, int K, int Nimg, int H, int W)
{
    if (dtype != NSK_BF16 || U != 4 || K != 64 || hooks().no_stem_halo) return false;
    const int PW = W + 3;
    if (SH_T + 3 * (PW + 1) > SH_MAX_IN) return false;
    const long long pi = (long long)(H + 3) * PW, total = pi * Nimg;
    if (total >= (1LL << 30) || total * pi >= (1LL << 40)) return false;   // exactness of the reciprocal division
    if (total * 128 >= (long long)SH_OOB) return false;
    return true;
}

// backward = 0: src = x2 [Nimg][H][W][16], wpk = w2 [64][16 taps][16], out = y [Nimg][H][W][64]
// backward = 1: src = dy [Nimg][H][W][64], wpk = w2 [16][16 taps][64], out = dx2 [Nimg][H][W][16]
// umin = -2: the taps are u, v in [-2, 1]; the backward pass reads dy at pos - (u, v).
namespace {
constexpr int kStemStatsGrid = 512;   // block count when statistics are requested (independent of the device)
}

// Rows of partial sums the forward launch writes (4 per block).
int stem_halo_stats_rows(int Nimg, int H, int W)
{
    const int tiles = ceil_div((H + 3) * (W + 3) * Nimg, SH_T);
    return (tiles < kStemStatsGrid ? tiles : kStemStatsGrid) * 4;
}

int launch_stem_halo(int backward, const void *src, const void *wpk, void *out, int Nimg, int H, int W, float *stats,
                     int stats_rows, hipStream_t stream)
{
    StemHaloArgs a{};
    a.src = src; a.wpk = wpk; a.out = out;
    a.H = H; a.W = W;
    a.PW = W + 3; a.PI = (H + 3) * a.PW;
    a.padlo = backward ? 1 : 2;
    a.total_pos = a.PI * Nimg;
    a.tiles = ceil_div(a.total_pos, SH_T);
    a.halo_lo = (backward ? 1 : 2) * (a.PW + 1);
    a.halo_hi = (backward ? 2 : 1) * (a.PW + 1);
    a.magic_pi = ((1ULL << 40) + a.PI - 1) / a.PI;
    a.magic_pw = ((1ULL << 40) + a.PW - 1) / a.PW;
    const size_t pix = (size_t)Nimg * H * W;
    a.src_bytes = (unsigned)(pix * (backward ? 128 : 32));
    a.out_bytes = (unsigned)(pix * (backward ? 32 : 128));
    for (int t = 0; t < 16; ++t) {
        const int u = t / 4 - 2, v = t % 4 - 2;
        a.tapoff[t] = backward ? -(u * a.PW + v) : u * a.PW + v;
    }
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return NSK_ERR_HIP;
        cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    }
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)stem_halo_kernel<2, 2, 64>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           stem_halo_smem<2, 2, 64>());
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)stem_halo_kernel<8, 1, 16>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    stem_halo_smem<8, 1, 16>());
        if (e != hipSuccess) {
            set_last_hip_error(e);
            return NSK_ERR_HIP;
        }
        attr_set = true;
    }
    // two blocks per CU in the forward pass (65 KB of LDS each): one block's epilogue overlaps the other's MFMAs
    const int want = backward ? cus : (stats ? kStemStatsGrid : 2 * cus);
    const int grid = a.tiles < want ? a.tiles : want;
    if (stats && (backward || stats_rows != grid * 4)) return NSK_ERR_BAD_DESC;   // the planner and the launch disagree
    a.stats = stats;
    a.stats_rows = stats_rows;
    const int smem_b = stem_halo_smem<8, 1, 16>(), smem_f = stem_halo_smem<2, 2, 64>();
    if (backward)
        hipLaunchKernelGGL((stem_halo_kernel<8, 1, 16>), dim3(grid), dim3(256), smem_b, stream, a);
    else
        hipLaunchKernelGGL((stem_halo_kernel<2, 2, 64>), dim3(grid), dim3(256), smem_f, stream, a);
    return check_launch();
}

}  // namespace nsk

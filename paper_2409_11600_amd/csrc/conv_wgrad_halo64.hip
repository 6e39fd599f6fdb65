// Backward-weight for the 3x3, stride 1, 64 -> 64 channel layers (fp32 and bf16): the weight gradient
// the paper accumulates into its gradient cache (section "Caching and Pooling"), for the layer shape
// that carries most of the 3x3 FLOPs of the residual networks it trains.
//
// dw[k][tap][c] = sum over positions q of dy[q][k] * x[q + shift(tap)][c].  As in the forward halo
// kernel, x and dy are addressed in flat zero-padded coordinates (every image a (H+2) x (W+2) grid,
// all images end to end), so a tap is one constant shift, padding positions load zeros through
// out-of-range buffer offsets, and the reduction simply runs over consecutive positions.
//
// A block walks over chunks of P consecutive positions.  Per chunk it stages dy[P][64] and
// x[P + 2*halo][64] ONCE in LDS (natural position-major layout) and all nine taps read the x tile at
// shifted rows; the 64 x 576 result lives in registers for the life of the block (2 x 18 accumulator
// tiles of 32x32 over 4 wavefronts: each wavefront both row halves and 5 (or 4) of the 18 column
// tiles) and is written once, as a float partial that wgrad_reduce_kernel combines in fixed order.
//
// The reduction index (position) is the slow index of both operands.  fp32 (mfma 32x32x2, one k per
// lane) reads that layout directly.  bf16 (mfma 32x32x16, 8 consecutive k per lane) uses the gfx950
// transposing LDS read (ds_read_b64_tr_b16): lanes 4j..4j+3 of a 16-lane group address row j (16
// consecutive channels) and lane i receives channel i of the four rows, i.e. four consecutive
// positions of one channel; rows are padded to 192 bytes so that the four rows read by each of two
// neighbouring 16-lane groups fall into eight different 32-byte bank groups of the 64-bank LDS.
#include <stdlib.h>

#include "nsk_internal.h"

namespace nsk {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr unsigned WH_OOB = 0xF0000000u;
constexpr int WH_MAX_HALO = 64;

struct WHArgs {
    const void *x, *dy;
    float *part;  // [blocks][64][9][64]
    int PW, PI, H, W;
    int total_pos, chunks, chunks_per_block, halo;
    unsigned long long magic_pi, magic_pw;
    unsigned bytes;  // size of x (= size of dy)
    int tapoff[9];
};

template <typename T> struct WH;
template <> struct WH<float> {
    static constexpr int P = 64, ROW = 256, VPP = 16, FRAG_COL = 128;
};
template <> struct WH<bf16_t> {
    static constexpr int P = 128, ROW = 192, VPP = 8, FRAG_COL = 64;
};

// SPLIT: eight wavefronts with split roles.  Wavefronts 0-3 only multiply; wavefronts 4-7 only move data: while chunk c
// is multiplied out of one LDS buffer they load chunk c + 1 and write it to the other, so staging (global loads, LDS
// writes, the address arithmetic) no longer sits between two runs of MFMAs of the same wavefront.  One barrier per chunk.
template <typename T, bool SPLIT>
__global__ __launch_bounds__(SPLIT ? 512 : 256) void wgrad_halo64_kernel(const WHArgs a)
{
    typedef WH<T> C;
    constexpr bool F32 = sizeof(T) == 4;
    constexpr int P = C::P, ROW = C::ROW, VPP = C::VPP;
    constexpr int XMAX = P + 2 * WH_MAX_HALO;
    constexpr int XL = XMAX * VPP / 256, DL = P * VPP / 256;
    constexpr int BUF = (XMAX + P) * ROW;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned *in_tab = (unsigned *)(smem + 2 * BUF);  // [2][XMAX]

    const int tid = threadIdx.x & 255, lane = tid & 63, wave = tid >> 6;   // index within the role
    const bool mover = SPLIT && threadIdx.x >= 256;
    const int frow = lane & 31, fk = lane >> 5;
    const __amdgpu_buffer_rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, a.bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t dy_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.dy, 0, a.bytes, 0x00020000);
    const int xn = P + 2 * a.halo;

    auto src_offset = [&](int q) -> unsigned {
        const bool inside = (unsigned)q < (unsigned)a.total_pos;
        const unsigned qq = inside ? (unsigned)q : 0u;
        const unsigned img = (unsigned)(((unsigned long long)qq * a.magic_pi) >> 40);
        const unsigned rem = qq - img * (unsigned)a.PI;
        const unsigned hp = (unsigned)(((unsigned long long)rem * a.magic_pw) >> 40);
        const unsigned wp = rem - hp * (unsigned)a.PW;
        const bool ok = inside & (hp - 1u < (unsigned)a.H) & (wp - 1u < (unsigned)a.W);
        const unsigned off = (((img * a.H + (hp - 1u)) * a.W + (wp - 1u)) * 64u) * (unsigned)sizeof(T);
        return ok ? off : WH_OOB;
    };
    auto fill_tab = [&](int chunk, int which) {
        if (tid < XMAX) in_tab[which * XMAX + tid] = tid < xn ? src_offset(chunk * P - a.halo + tid) : WH_OOB;
    };

    u32x4 stage[XL + DL];
    auto issue_loads = [&](int which) {
        const unsigned *tab = in_tab + which * XMAX;
#pragma unroll
        for (int u = 0; u < XL; ++u) {
            const int idx = tid + 256 * u, pos = idx / VPP, v = idx % VPP;
            const unsigned off = tab[pos];
            stage[u] = __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, off == WH_OOB ? WH_OOB : off + v * 16, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < DL; ++u) {
            const int idx = tid + 256 * u, pos = idx / VPP, v = idx % VPP;
            const unsigned off = tab[a.halo + pos];
            stage[XL + u] = __builtin_amdgcn_raw_buffer_load_b128(dy_rsrc, off == WH_OOB ? WH_OOB : off + v * 16, 0, 0);
        }
    };
    // the same loads with every lane computing its own source offsets (the moving wavefronts have the time, and
    // no table means no barrier among them)
    auto issue_loads_direct = [&](int chunk) {
#pragma unroll
        for (int u = 0; u < XL; ++u) {
            const int idx = tid + 256 * u, pos = idx / VPP, v = idx % VPP;
            const unsigned off = pos < xn ? src_offset(chunk * P - a.halo + pos) : WH_OOB;
            stage[u] = __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, off == WH_OOB ? WH_OOB : off + v * 16, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < DL; ++u) {
            const int idx = tid + 256 * u, pos = idx / VPP, v = idx % VPP;
            const unsigned off = src_offset(chunk * P + pos);
            stage[XL + u] = __builtin_amdgcn_raw_buffer_load_b128(dy_rsrc, off == WH_OOB ? WH_OOB : off + v * 16, 0, 0);
        }
    };
    auto write_stage = [&](unsigned char *buf) {
#pragma unroll
        for (int u = 0; u < XL; ++u) {
            const int idx = tid + 256 * u, pos = idx / VPP, v = idx % VPP;
            *(u32x4 *)(buf + pos * ROW + v * 16) = stage[u];
        }
#pragma unroll
        for (int u = 0; u < DL; ++u) {
            const int idx = tid + 256 * u, pos = idx / VPP, v = idx % VPP;
            *(u32x4 *)(buf + (XMAX + pos) * ROW + v * 16) = stage[XL + u];
        }
    };

    const int c_begin = blockIdx.x * a.chunks_per_block;
    const int c_end = min(a.chunks, c_begin + a.chunks_per_block);
    if (mover) {
        // The moving wavefronts' whole life (kept apart from the multiplying code so that the accumulators are not live
        // here): one barrier after the first chunk is in place, one at the end of every chunk, as on the other side.
        if (c_begin < c_end) {
            issue_loads_direct(c_begin);
            write_stage(smem);
            __syncthreads();
        }
        for (int c = c_begin; c < c_end; ++c) {
            const int cur = (c - c_begin) & 1;
            // the other buffer was last read before the barrier that ended the previous chunk
            if (c + 1 < c_end) {
                issue_loads_direct(c + 1);
                write_stage(smem + (cur ^ 1) * BUF);
            }
            __syncthreads();
        }
        return;
    }

    // column tiles of this wavefront: nf = wave + 4*ni (tap = nf/2, channel half = nf%2); the fifth
    // one of wavefronts 2 and 3 does not exist: it computes on tap 0 and is never stored.
    int n_tap[5], n_half[5];
    unsigned n_base[5];
#pragma unroll
    for (int ni = 0; ni < 5; ++ni) {
        const int nf = wave + 4 * ni;
        n_tap[ni] = nf < 18 ? nf >> 1 : 0;
        n_half[ni] = nf < 18 ? nf & 1 : 0;
        n_base[ni] = (unsigned)((a.halo + a.tapoff[n_tap[ni]]) * ROW + n_half[ni] * C::FRAG_COL);
    }
    // per-lane offset of a fragment element inside a tile (see the header comment)
    unsigned lane_off;
    if (F32) {
        lane_off = (unsigned)(fk * ROW + frow * 4);
    } else {
        const int g = lane >> 4, i16 = lane & 15;
        lane_off = (unsigned)((8 * (g >> 1) + (i16 >> 2)) * ROW + (16 * (g & 1) + 4 * (i16 & 3)) * 2);
    }

    f32x16 acc[2][5];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 5; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

    if (SPLIT) {
        if (c_begin < c_end) __syncthreads();   // the first chunk is in place
    } else if (c_begin < c_end) {
        fill_tab(c_begin, 0);
        __syncthreads();
        issue_loads(0);
    }
    for (int c = c_begin; c < c_end; ++c) {
        const int cur = (c - c_begin) & 1;
        unsigned char *buf = smem + cur * BUF;
        if (!SPLIT) {
            write_stage(buf);
            if (c + 1 < c_end) fill_tab(c + 1, cur ^ 1);
            __syncthreads();
            if (c + 1 < c_end) issue_loads(cur ^ 1);   // lands in registers while this chunk is computed
        }

        const unsigned char *xb = buf + lane_off;
        const unsigned char *db = buf + XMAX * ROW + lane_off;
        if constexpr (F32) {
#pragma unroll 4
            for (int s = 0; s < P / 2; ++s) {
                float av[2], bv[5];
#pragma unroll
                for (int mi = 0; mi < 2; ++mi) av[mi] = *(const float *)(db + 2 * s * ROW + mi * 128);
#pragma unroll
                for (int ni = 0; ni < 5; ++ni) bv[ni] = *(const float *)(xb + n_base[ni] + 2 * s * ROW);
#pragma unroll
                for (int ni = 0; ni < 5; ++ni)
#pragma unroll
                    for (int mi = 0; mi < 2; ++mi)
                        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[mi], bv[ni], acc[mi][ni], 0, 0, 0);
            }
        } else {
            typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
            auto tr8 = [&](const unsigned char *p) -> bf16x8 {
                // 8 consecutive positions of this lane's channel: two transposing reads of 4 rows each
                const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)(p));
                const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)(p + 4 * ROW));
                bf16x8 r;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    r[e] = lo[e];
                    r[4 + e] = hi[e];
                }
                return r;
            };
            bf16x8 af[2][2], bq[2][5];
            auto fetch = [&](int s, int set) {
#pragma unroll
                for (int mi = 0; mi < 2; ++mi) af[set][mi] = tr8(db + 16 * s * ROW + mi * 64);
#pragma unroll
                for (int ni = 0; ni < 5; ++ni) bq[set][ni] = tr8(xb + n_base[ni] + 16 * s * ROW);
            };
            fetch(0, 0);
#pragma unroll
            for (int s = 0; s < P / 16; ++s) {
                if (s + 1 < P / 16) fetch(s + 1, (s + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int ni = 0; ni < 5; ++ni)
#pragma unroll
                    for (int mi = 0; mi < 2; ++mi)
                        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[s & 1][mi], bq[s & 1][ni], acc[mi][ni], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (SPLIT) __syncthreads();   // the chunk is consumed and the next one is in place
    }

    // acc[mi][ni][v]: row k = 32*mi + 8*(v/4) + 4*(lane/32) + v%4, column c = 32*half + lane%32
    float *__restrict__ part = a.part + (long)blockIdx.x * 64 * 9 * 64;
#pragma unroll
    for (int ni = 0; ni < 5; ++ni) {
        if (wave + 4 * ni >= 18) continue;
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = 32 * mi + 8 * (v >> 2) + 4 * fk + (v & 3);
                part[(k * 9 + n_tap[ni]) * 64 + n_half[ni] * 32 + frow] = acc[mi][ni][v];
            }
    }
}

// ------------------------------------------------------------------------------------------------
// fp32, images 32 pixels wide: ROW-ALIGNED chunks.  A chunk is two rows of one image (64 real output
// pixels, contiguous in memory for dy); x is staged as the four rows around them, each with its two
// padding columns (4 x 34 positions).  No matrix work goes to padding positions, N*H/2 chunks divide
// evenly over the blocks for the configured batches, and every LDS offset is a compile-time constant.
// Each wavefront owns one half of the output channels k and one half of the input channels c for all
// nine taps: 9 accumulator tiles, perfectly balanced.
constexpr int R32_W = 32, R32_PW = 34;
constexpr int R32_XPOS = 4 * R32_PW;   // 136 staged x positions
constexpr int R32_ROW = 256;           // bytes per position (64 floats)
constexpr int R32_BUF = (R32_XPOS + 64) * R32_ROW;
constexpr int R32_XL = (R32_XPOS * 16 + 255) / 256;   // 9 x vectors per thread (the last pass is partial)

struct WR32Args {
    const void *x, *dy;
    const float *act;   // nullptr, or [2][64]: x is relu(act[c]*x + act[64+c]), applied while a chunk is staged
    float *part;
    int H, PI, chunks_per_img, chunks, chunks_per_block, total_pos;
    unsigned long long magic_pi;
    unsigned bytes;
};

template <bool ACT>
__global__ __launch_bounds__(256) void wgrad_rows32_f32_kernel(const WR32Args a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int frow = lane & 31, fk = lane >> 5;
    const int mi = wave & 1, ch = wave >> 1;
    const __amdgpu_buffer_rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, a.bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t dy_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a.dy, 0, a.bytes, 0x00020000);

    // staged x position p of chunk (img, h0): padded row h0 + p/34 (real row h0 - 1 + p/34), padded column p%34
    u32x4 stage[R32_XL + 4];
    // ACT: a thread always stages the same four channels of x (4*(tid%16) ..); one bit per pass marks real positions
    float asc[4] = {0.f, 0.f, 0.f, 0.f}, ash[4] = {0.f, 0.f, 0.f, 0.f};
    if (ACT) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            asc[e] = a.act[(tid & 15) * 4 + e];
            ash[e] = a.act[64 + (tid & 15) * 4 + e];
        }
    }
    unsigned real_bits = 0;
    auto issue_loads = [&](int chunk) {
        const int img = chunk / a.chunks_per_img, h0 = (chunk % a.chunks_per_img) * 2;
        real_bits = 0;
#pragma unroll
        for (int u = 0; u < R32_XL; ++u) {
            const int idx = tid + 256 * u, p = idx >> 4, v = idx & 15;
            const int pr = p / R32_PW, pc = p - pr * R32_PW;
            const int h = h0 - 1 + pr, w = pc - 1;
            const bool ok = p < R32_XPOS && (unsigned)h < (unsigned)a.H && (unsigned)w < (unsigned)R32_W;
            const unsigned off = (unsigned)((((img * a.H + h) * R32_W + w) * 64 + v * 4) * 4);
            stage[u] = __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, ok ? off : WH_OOB, 0, 0);
            if (ACT) real_bits |= (ok ? 1u : 0u) << u;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = tid + 256 * u;   // 64 pixels x 16 vectors, contiguous in memory
            stage[R32_XL + u] = __builtin_amdgcn_raw_buffer_load_b128(
                dy_rsrc, (unsigned)(((img * a.H + h0) * R32_W * 64 + idx * 4) * 4), 0, 0);
        }
    };
    auto write_stage = [&](unsigned char *buf) {
#pragma unroll
        for (int u = 0; u < R32_XL; ++u) {
            const int idx = tid + 256 * u;
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
            if (idx < R32_XPOS * 16) *(u32x4 *)(buf + idx * 16) = stage[u];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) *(u32x4 *)(buf + R32_XPOS * R32_ROW + (tid + 256 * u) * 16) = stage[R32_XL + u];
    };

    f32x16 acc[9];
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;

    const int c_begin = blockIdx.x * a.chunks_per_block;
    const int c_end = min(a.chunks, c_begin + a.chunks_per_block);
    if (c_begin < c_end) issue_loads(c_begin);
    const unsigned a_lane = (unsigned)(R32_XPOS * R32_ROW + fk * R32_ROW + (32 * mi + frow) * 4);
    const unsigned b_lane = (unsigned)(fk * R32_ROW + (32 * ch + frow) * 4);
    for (int c = c_begin; c < c_end; ++c) {
        unsigned char *buf = smem + ((c - c_begin) & 1) * R32_BUF;
        write_stage(buf);
        __syncthreads();
        if (c + 1 < c_end) issue_loads(c + 1);
#pragma unroll
        for (int s = 0; s < 32; ++s) {
            // output pixels 2s, 2s+1 of the chunk: row r = s/16, columns (2s)%32 + {0,1}
            const int r = s >> 4, col = (2 * s) & 31;
            const float av = *(const float *)(buf + a_lane + 2 * s * R32_ROW);
            float bv[9];
#pragma unroll
            for (int t = 0; t < 9; ++t)
                bv[t] = *(const float *)(buf + b_lane + ((r + t / 3) * R32_PW + col + t % 3) * R32_ROW);
#pragma unroll
            for (int t = 0; t < 9; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv[t], acc[t], 0, 0, 0);
        }
    }
    float *__restrict__ part = a.part + (long)blockIdx.x * 64 * 9 * 64;
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int k = 32 * mi + 8 * (v >> 2) + 4 * fk + (v & 3);
            part[(k * 9 + t) * 64 + ch * 32 + frow] = acc[t][v];
        }
}

bool rows32_f32(int dtype, const WgradArgs &a) { return dtype == NSK_F32 && a.W == R32_W && a.H % 2 == 0; }
}  // namespace

// True if the kernel launch_wgrad_halo64 picks applies WgradArgs::act while it stages x.
bool wgrad_halo64_act_fused(int dtype, const WgradArgs &a) { return wgrad_halo64_applicable(dtype, a) && rows32_f32(dtype, a); }

namespace {

template <typename T> int smem_bytes()
{
    constexpr int XMAX = WH<T>::P + 2 * WH_MAX_HALO;
    return 2 * (XMAX + WH<T>::P) * WH<T>::ROW + 2 * XMAX * 4;
}

}  // namespace

// Geometry test shared by the workspace planner and the launcher (host only, no HIP calls).
bool wgrad_halo64_applicable(int dtype, const WgradArgs &a)
{
    if (a.C != 64 || a.K != 64 || a.ntaps != 9) return false;
    if (a.sh != 1 || a.sw != 1 || a.ph != 1 || a.pw != 1 || a.P != a.H || a.Q != a.W) return false;
    for (int t = 0; t < 9; ++t)
        if (a.off_h[t] != t / 3 || a.off_w[t] != t % 3) return false;
    if (a.W + 3 > WH_MAX_HALO) return false;
    const long long pi = (long long)(a.H + 2) * (a.W + 2), total = pi * a.Nimg;
    if (total >= (1LL << 30) || total * pi >= (1LL << 40)) return false;
    const unsigned long long bytes = (unsigned long long)a.Nimg * a.H * a.W * 64 * (dtype == NSK_BF16 ? 2 : 4);
    if (bytes >= WH_OOB) return false;
    return true;
}

// Number of float partials ([64][9][64] each) the launcher will write: at most one per CU.
int wgrad_halo64_partials(int dtype, const WgradArgs &a, int *chunks_per_block)
{
    const int P = dtype == NSK_BF16 ? WH<bf16_t>::P : WH<float>::P;
    const long long total = (long long)(a.H + 2) * (a.W + 2) * a.Nimg;
    int chunks = (int)((total + P - 1) / P);
    if (rows32_f32(dtype, a)) chunks = a.Nimg * (a.H / 2);   // row-aligned chunks of two image rows
    int grid = chunks < 256 ? chunks : 256;
    // Every block writes a whole [64][9][64] float partial (147 KB) that the reduction reads again, so a small problem
    // is not spread over more blocks than gives each two chunks (measured, bf16 8x8 images, batch 256: 23.5 -> 18.8 us;
    // fp32 chunks are half as long and lose)
    if (dtype == NSK_BF16 && !rows32_f32(dtype, a) && chunks / 2 < grid) grid = chunks / 2 > 0 ? chunks / 2 : 1;
    const int cpb = (chunks + grid - 1) / grid;
    if (chunks_per_block) *chunks_per_block = cpb;
    return (chunks + cpb - 1) / cpb;
}

int launch_wgrad_halo64(int dtype, const WgradArgs &g, hipStream_t stream)
{
    if (((uintptr_t)g.x | (uintptr_t)g.dy) & 15) return NSK_ERR_ALIGNMENT;
    if (rows32_f32(dtype, g)) {
        WR32Args r{};
        r.x = g.x; r.dy = g.dy; r.part = g.part;
        r.H = g.H;
        r.chunks_per_img = g.H / 2;
        r.chunks = g.Nimg * r.chunks_per_img;
        const int blocks = wgrad_halo64_partials(dtype, g, &r.chunks_per_block);
        r.bytes = (unsigned)((size_t)g.Nimg * g.H * g.W * 64 * 4);
        static bool r_attr = false;
        if (!r_attr) {
            hipError_t e = hipFuncSetAttribute((const void *)wgrad_rows32_f32_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * R32_BUF);
            if (e == hipSuccess)
                e = hipFuncSetAttribute((const void *)wgrad_rows32_f32_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * R32_BUF);
            if (e != hipSuccess) {
                set_last_hip_error(e);
                return NSK_ERR_HIP;
            }
            r_attr = true;
        }
        r.act = g.act;
        if (g.act)
            hipLaunchKernelGGL(wgrad_rows32_f32_kernel<true>, dim3(blocks), dim3(256), 2 * R32_BUF, stream, r);
        else
            hipLaunchKernelGGL(wgrad_rows32_f32_kernel<false>, dim3(blocks), dim3(256), 2 * R32_BUF, stream, r);
        return check_launch();
    }
    if (g.act) return NSK_ERR_BAD_DESC;   // only the row-aligned fp32 kernel above applies the activation on load
    WHArgs a{};
    a.x = g.x; a.dy = g.dy; a.part = g.part;
    a.H = g.H; a.W = g.W;
    a.PW = g.W + 2; a.PI = (g.H + 2) * a.PW;
    a.total_pos = a.PI * g.Nimg;
    const int P = dtype == NSK_BF16 ? WH<bf16_t>::P : WH<float>::P;
    a.chunks = ceil_div(a.total_pos, P);
    const int blocks = wgrad_halo64_partials(dtype, g, &a.chunks_per_block);
    a.halo = a.PW + 1;
    a.magic_pi = ((1ULL << 40) + a.PI - 1) / a.PI;
    a.magic_pw = ((1ULL << 40) + a.PW - 1) / a.PW;
    a.bytes = (unsigned)((size_t)g.Nimg * g.H * g.W * 64 * (dtype == NSK_BF16 ? 2 : 4));
    for (int t = 0; t < 9; ++t) a.tapoff[t] = (t / 3 - 1) * a.PW + (t % 3 - 1);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)wgrad_halo64_kernel<float, false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           smem_bytes<float>());
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)wgrad_halo64_kernel<bf16_t, false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    smem_bytes<bf16_t>());
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)wgrad_halo64_kernel<float, true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    smem_bytes<float>());
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)wgrad_halo64_kernel<bf16_t, true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    smem_bytes<bf16_t>());
        if (e != hipSuccess) {
            set_last_hip_error(e);
            return NSK_ERR_HIP;
        }
        attr_set = true;
    }
    const bool split = !hooks().wh_no_split;   // the variable is an A/B and test hook
    if (dtype == NSK_BF16) {
        if (split)
            hipLaunchKernelGGL((wgrad_halo64_kernel<bf16_t, true>), dim3(blocks), dim3(512), smem_bytes<bf16_t>(), stream, a);
        else
            hipLaunchKernelGGL((wgrad_halo64_kernel<bf16_t, false>), dim3(blocks), dim3(256), smem_bytes<bf16_t>(), stream, a);
    } else {
        if (split)
            hipLaunchKernelGGL((wgrad_halo64_kernel<float, true>), dim3(blocks), dim3(512), smem_bytes<float>(), stream, a);
        else
            hipLaunchKernelGGL((wgrad_halo64_kernel<float, false>), dim3(blocks), dim3(256), smem_bytes<float>(), stream, a);
    }
    return check_launch();
}

}  // namespace nsk

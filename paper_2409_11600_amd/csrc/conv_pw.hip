// Short-reduction convolution for bf16 layers whose whole reduction fits in a lane's registers: one, two, four or
// nine taps of 16 to 256 channels, at most 256 reduction indices (288 / 576 for a 3x3 filter on 32 / 64 channels).
// These are the 1x1 layers of a bottleneck block in both directions, the residue classes of the backward-data pass
// of a stride-2 layer, the strided 3x3 64 -> 64 layer, and every 16- and 32-channel layer of the CIFAR-sized network
// of the ResNet recipe the paper trains (section "Experiments and Discussion").
//
// Such layers move about ten times more bytes per multiply than the matrix units need (or are so small that every
// kernel is latency-bound), so the kernel is built around the memory stream and not around the multiply:
//   * the whole filter ([Ngemm][taps][Cs], at most 74 KB) is copied to LDS once per block and stays there;
//   * a wavefront owns a tile of 32*FM pixels and loads their channels straight into registers in the MFMA
//     operand layout (lane = pixel, 16 bytes = 8 consecutive channels): the activations never pass through LDS;
//   * the loads of the next tile are issued before the current tile is multiplied, so every wavefront keeps a
//     whole tile of loads in flight while it multiplies, converts and stores;
//   * wavefronts never wait for each other after the filter copy (no barrier in the tile loop);
//   * output channels are handled in chunks of NW (64, or a whole 32- or 16-channel output), staged through a
//     per-wavefront LDS strip so that a pixel's chunk leaves as 16-byte pieces of contiguous lanes;
//   * an accumulating launch fetches the old output values the same way, one chunk ahead, and adds them to the
//     fp32 sums before the single rounding;
//   * a forward launch can leave per-channel partial sums for the batch-norm behind it, and the launch for the one
//     live class of a 1x1 stride-2 backward-data pass also writes the zeros of the other three pixels of each cell.
// One block of 4 wavefronts per CU (the register file then allows two tiles of up to 256 channels per lane);
// 256 persistent blocks.  This file holds the 64-channel-chunk instances, conv_pw_narrow16/32.hip the narrow ones.
#include "conv_pw_kernel.h"

namespace nsk {

bool conv_pw_applicable(int dtype, const IgemmArgs &a)
{
    if (hooks().no_pw) return false;
    if (dtype != NSK_BF16 || (a.accumulate && (a.stats || a.zero_cell))) return false;
    if (a.Cs % 16 != 0 || a.Ktot != a.ntaps * a.Cs) return false;
    const int ks = a.Ktot / 16;
    long min_rows;
    if (a.Ngemm == 16 || a.Ngemm == 32) {
        // narrow outputs (the CIFAR-sized network): every kernel is latency-bound there and this one has the least set-up
        if (!conv_pw_narrow_instance(ks, a.ntaps)) return false;
        min_rows = 8192;
    } else if (a.Ngemm % 64 == 0) {
        if (a.ntaps == 9) {
            // a whole 3x3 filter on 64 (or 32) -> 64 channels; the stride-1 64 -> 64 layer has a kernel that reuses the halo
            if (!(a.Cs == 64 || a.Cs == 32) || a.Ngemm != 64 || (a.Cs == 64 && a.mult_h == 1 && a.mult_w == 1)) return false;
        } else {
            if (!(a.ntaps == 1 || a.ntaps == 2 || a.ntaps == 4)) return false;
            // (512 channels in one tap: 128 registers per lane and tile, two tiles in flight)
            if (!(a.Cs == 64 || a.Cs == 128 || a.Cs == 256 || ((a.Cs == 32 || a.Cs == 512) && a.ntaps == 1)) || (a.Ktot > 256 && a.Cs != 512))
                return false;
        }
        const int cols = pw_cols(a);
        if (cols == 0) return false;
        // enough tiles to give every wavefront of the grid a few (below that the generic kernel's many small blocks
        // win); with the columns split into groups every group walks over all rows, so fewer rows are enough
        min_rows = a.Cs == 32 ? 8192 : (4L * kPwGrid * 4 * 64) / ((a.Ngemm / cols) * (a.Ngemm / cols));
    } else {
        return false;
    }
    if (a.Co % 8 != 0 || (uintptr_t)a.out % 16 != 0 || (uintptr_t)a.src % 16 != 0 || (uintptr_t)a.wpk % 16 != 0) return false;
    // 32-bit byte offsets below the out-of-range marker
    if ((long)a.Nimg * a.Ho * a.Wo * a.Co * 2 >= (long)PW_OOB || (long)a.src_bytes >= (long)PW_OOB) return false;
    // exact magic-number division of a row index by Mi*Mj and of the remainder by Mj
    if ((long)a.M * a.Mi * a.Mj >= (1L << 40) || (long)a.Mi * a.Mj * a.Mj >= (1L << 40)) return false;
    if (hooks().pw_min_rows >= 0) min_rows = (long)hooks().pw_min_rows;   // test hook
    return a.M >= min_rows;
}

// one row per wavefront of every row share (the column groups of a split output write different columns of a row)
int conv_pw_stats_rows(const IgemmArgs &a)
{
    const int cols = pw_cols(a);
    return cols > 0 ? kPwGrid * 4 / (a.Ngemm / cols) : kPwGrid * 4;
}

int launch_conv_pw(const IgemmArgs &a, hipStream_t stream)
{
    PwArgs pa;
    pa.g = a;
    pa.tiles = 0;   // set by the launcher that knows the tile height
    pa.zero_cell = a.zero_cell;
    pa.out_bytes = (unsigned)((long)a.Nimg * a.Ho * a.Wo * a.Co * 2);
    const unsigned long long one = 1ull << 40;
    const unsigned long long per_img = (unsigned long long)a.Mi * a.Mj;
    pa.magic_img = (one + per_img - 1) / per_img;
    pa.magic_row = (one + a.Mj - 1) / a.Mj;
    if (pw_chunk(a) == 16) return launch_conv_pw_narrow16(pa, stream);
    if (pw_chunk(a) == 32) return launch_conv_pw_narrow32(pa, stream);
    switch (a.Ktot / 16 * 16 + a.ntaps) {   // (k-steps, taps)
    case 4 * 16 + 1: return launch_pw<4, 2, 1, 64>(pa, stream);
    case 8 * 16 + 1: return launch_pw<8, 2, 1, 64>(pa, stream);
    case 8 * 16 + 2: return launch_pw<8, 2, 2, 64>(pa, stream);
    case 16 * 16 + 1: return launch_pw<16, 1, 1, 64>(pa, stream);
    case 16 * 16 + 2: return launch_pw<16, 1, 2, 64>(pa, stream);
    case 16 * 16 + 4: return launch_pw<16, 1, 4, 64>(pa, stream);
    case 36 * 16 + 9: return launch_pw<36, 1, 9, 64>(pa, stream);
    case 32 * 16 + 1: return launch_pw<32, 1, 1, 64>(pa, stream);    // 512 channels, one tap
    case 2 * 16 + 1: return launch_pw<2, 2, 1, 64>(pa, stream);      // 32 -> 64 channels, one tap
    case 18 * 16 + 9: return launch_pw<18, 2, 9, 64>(pa, stream);    // 32 -> 64 channels, 3x3
    default: return NSK_ERR_UNSUPPORTED;
    }
}

}  // namespace nsk

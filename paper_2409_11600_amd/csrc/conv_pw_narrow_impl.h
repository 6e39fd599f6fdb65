// Instances of the short-reduction convolution kernel for outputs of PW_NARROW_NW channels (16 or 32): the layers of
// the CIFAR-sized network of the ResNet recipe (section "Experiments and Discussion"), whose 16- and 32-channel
// convolutions are far too small for the tiled kernels' per-block set-up to pay off.  Included by
// conv_pw_narrow16.hip and conv_pw_narrow32.hip with PW_NARROW_NW defined.
#include "conv_pw_kernel.h"

namespace nsk {

#define PW_CAT2(a, b) a##b
#define PW_CAT(a, b) PW_CAT2(a, b)

int PW_CAT(launch_conv_pw_narrow, PW_NARROW_NW)(const PwArgs &pa, hipStream_t stream)
{
    constexpr int NW = PW_NARROW_NW;
    const IgemmArgs &a = pa.g;
    switch (a.Ktot / 16 * 16 + a.ntaps) {   // (k-steps, taps); 64-pixel tiles except for the 256-index reductions
    case 1 * 16 + 1: return launch_pw<1, 2, 1, NW>(pa, stream);
    case 2 * 16 + 2: return launch_pw<2, 2, 2, NW>(pa, stream);
    case 4 * 16 + 4: return launch_pw<4, 2, 4, NW>(pa, stream);
    case 9 * 16 + 9: return launch_pw<9, 2, 9, NW>(pa, stream);
    case 2 * 16 + 1: return launch_pw<2, 2, 1, NW>(pa, stream);
    case 4 * 16 + 2: return launch_pw<4, 2, 2, NW>(pa, stream);
    case 8 * 16 + 4: return launch_pw<8, 2, 4, NW>(pa, stream);
    case 18 * 16 + 9: return launch_pw<18, 2, 9, NW>(pa, stream);
    case 4 * 16 + 1: return launch_pw<4, 2, 1, NW>(pa, stream);
    case 8 * 16 + 2: return launch_pw<8, 2, 2, NW>(pa, stream);
    case 16 * 16 + 4: return launch_pw<16, 1, 4, NW>(pa, stream);
    default: return NSK_ERR_UNSUPPORTED;
    }
}

}  // namespace nsk

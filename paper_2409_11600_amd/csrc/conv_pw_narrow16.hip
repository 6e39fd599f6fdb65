// 16-channel outputs of the short-reduction convolution kernel (see conv_pw_narrow_impl.h).
#define PW_NARROW_NW 16
#include "conv_pw_narrow_impl.h"

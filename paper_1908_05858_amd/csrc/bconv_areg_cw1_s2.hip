// Activation-stationary binary convolution kernels: 1 packed 64-bit word per pixel, stride 2.
#include "bconv_areg_kernel.h"

namespace dabnn {
DABNN_DEFINE_AREG_ENTRY_POINTS(1, 2)
}  // namespace dabnn

// Activation-stationary binary convolution kernels: 7 packed 64-bit words per pixel, stride 1.
#include "bconv_areg_kernel.h"

namespace dabnn {
DABNN_DEFINE_AREG_ENTRY_POINTS(7, 1)
}  // namespace dabnn

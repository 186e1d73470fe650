// Activation-stationary binary convolution kernels: 3 packed 64-bit words per pixel, stride 2.
#include "bconv_areg_kernel.h"

namespace dabnn {
DABNN_DEFINE_AREG_ENTRY_POINTS(3, 2)
}  // namespace dabnn

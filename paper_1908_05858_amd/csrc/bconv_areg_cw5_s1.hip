// Activation-stationary binary convolution kernels: 5 packed 64-bit words per pixel, stride 1.
#include "bconv_areg_kernel.h"

namespace dabnn {
DABNN_DEFINE_AREG_ENTRY_POINTS(5, 1)
}  // namespace dabnn

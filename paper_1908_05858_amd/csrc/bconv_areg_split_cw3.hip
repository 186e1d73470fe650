// Activation-stationary binary convolution kernels in which the four wavefronts of a workgroup
// share a channel group: 3 packed 64-bit words per pixel and wavefront (12 per launch).
#include "bconv_areg_split_kernel.h"

namespace dabnn {
DABNN_DEFINE_SPLIT_ENTRY_POINT(3, )
}  // namespace dabnn

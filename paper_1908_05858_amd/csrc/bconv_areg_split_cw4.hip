// Activation-stationary binary convolution kernels in which the four wavefronts of a workgroup
// share a channel group: 4 packed 64-bit words per pixel and wavefront (16 per launch).
#include "bconv_areg_split_kernel.h"

namespace dabnn {
// (a tensor of exactly 16 words per pixel takes the instantiation with compile-time filter strides)
DABNN_DEFINE_SPLIT_ENTRY_POINT(4, if (cw_total == 16 && word0 == 0 && active_waves == 4)
                                      return launch_split_inst<4, false, false, 16>(L, s, stream);)
}  // namespace dabnn

// Activation-stationary binary convolution kernels in which the four wavefronts of a workgroup
// share a channel group: 1 packed 64-bit word per pixel and wavefront (4 per launch).
#include "bconv_areg_split_kernel.h"

namespace dabnn {
DABNN_DEFINE_SPLIT_ENTRY_POINT(1, if (active_waves < 4)
            return launch_split_inst<1, true>(L, s, stream);)
}  // namespace dabnn

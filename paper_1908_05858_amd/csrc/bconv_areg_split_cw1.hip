// Activation-stationary binary convolution kernels in which the four wavefronts of a workgroup
// share a channel group: 1 packed 64-bit word per pixel and wavefront (4 per launch).
#include "bconv_areg_split_kernel.h"

namespace dabnn {
// (a tensor of exactly 4 words per pixel takes the instantiation with compile-time filter strides)
DABNN_DEFINE_SPLIT_ENTRY_POINT(1, if (active_waves < 4)
            return launch_split_inst<1, true>(L, s, stream);
        if (cw_total == 4 && word0 == 0)
            return launch_split_inst<1, false, false, 4>(L, s, stream);)
}  // namespace dabnn

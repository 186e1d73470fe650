// Activation-stationary binary convolution kernels in which the four wavefronts of a workgroup
// share a channel group: 2 packed 64-bit words per pixel and wavefront (8 per launch).
#include "bconv_areg_split_kernel.h"

namespace dabnn {
// (a tensor of exactly 8 words per pixel, the Bi-Real-18 case, takes the instantiation with
// compile-time filter strides)
DABNN_DEFINE_SPLIT_ENTRY_POINT(2, if (cw_total == 8 && word0 == 0 && active_waves == 4)
                                      return launch_split_inst<2, false, false, 8>(L, s, stream);)

// 8 words per pixel with the fused threshold epilogue: one launch covers all words.
hipError_t launch_split_bits_cw2(const uint32_t* a, const uint32_t* w, uint64_t* out,
                                 const int32_t* thr, const uint64_t* flip, const ConvShape& s,
                                 hipStream_t stream)
{
    const SplitLaunch L{a, w, reinterpret_cast<int32_t*>(out), 8, 0, true, 4, thr, flip};
    return launch_split_inst<2, false, true, 8>(L, s, stream);
}
}  // namespace dabnn

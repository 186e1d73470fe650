// Dispatch of the activation-stationary binary convolution family (kernels: bconv_areg_kernel.h,
// instantiated per word count in bconv_areg_cw<Cw>.hip).
#include "launch.h"

namespace dabnn {

#define DABNN_DECLARE(CW, S)                                                                       \
    hipError_t launch_areg_cw##CW##_s##S(const uint32_t* a, const uint32_t* w, int32_t* y,         \
                                         const ConvShape& s, hipStream_t stream);                 \
    hipError_t launch_bits_cw##CW##_s##S(const uint32_t* a, const uint32_t* w, uint64_t* out,      \
                                         const ConvShape& s, hipStream_t stream,                  \
                                         const int32_t* thr, const uint2* flip);                  \
    hipError_t launch_res_cw##CW##_s##S(const uint32_t* a, const uint32_t* w, const ConvShape& s,  \
                                        hipStream_t stream, const float* scale,                   \
                                        const float* shift, const float* r, float* x_out,         \
                                        uint64_t* bits);
DABNN_DECLARE(1, 1) DABNN_DECLARE(1, 2) DABNN_DECLARE(2, 1) DABNN_DECLARE(2, 2)
DABNN_DECLARE(4, 1) DABNN_DECLARE(4, 2) DABNN_DECLARE(8, 1) DABNN_DECLARE(8, 2)
#undef DABNN_DECLARE

// The kernels address a window tap as the tensor base plus a 32-bit BYTE offset, and (on the
// direct-store path) the output with 32-bit element offsets: the packed activation tensor must
// stay below 4 GiB and the output below 2^31 elements.  Larger tensors run the other families,
// which index with size_t.
static bool areg_offsets_fit(const ConvShape& s)
{
    const int64_t act_bytes = static_cast<int64_t>(s.N) * s.H * s.W * s.Cw * 8;
    const int64_t out_elems = static_cast<int64_t>(s.N) * s.Ho * s.Wo * s.Cout;
    return act_bytes < (int64_t{1} << 32) && out_elems < (int64_t{1} << 31);
}

bool bconv_bnsign_areg_supports(const ConvShape& s)
{
    return areg_offsets_fit(s) && s.kh == 3 && s.kw == 3 && (s.stride == 1 || s.stride == 2) &&
           (s.Cw == 1 || s.Cw == 2 || s.Cw == 4 || s.Cw == 8) && s.Cout % 64 == 0;
}

hipError_t launch_bconv_bnsign_areg(const uint64_t* a, const uint64_t* w, const int32_t* thr,
                                    const uint64_t* flip, uint64_t* out, const ConvShape& s,
                                    hipStream_t stream)
{
    if (!bconv_bnsign_areg_supports(s))
        return hipErrorNotSupported;
    const uint32_t* a32 = reinterpret_cast<const uint32_t*>(a);
    const uint32_t* w32 = reinterpret_cast<const uint32_t*>(w);
    const uint2* f2 = reinterpret_cast<const uint2*>(flip);
    switch (s.Cw) {
        case 1:
            return s.stride == 1 ? launch_bits_cw1_s1(a32, w32, out, s, stream, thr, f2)
                                 : launch_bits_cw1_s2(a32, w32, out, s, stream, thr, f2);
        case 2:
            return s.stride == 1 ? launch_bits_cw2_s1(a32, w32, out, s, stream, thr, f2)
                                 : launch_bits_cw2_s2(a32, w32, out, s, stream, thr, f2);
        case 4:
            return s.stride == 1 ? launch_bits_cw4_s1(a32, w32, out, s, stream, thr, f2)
                                 : launch_bits_cw4_s2(a32, w32, out, s, stream, thr, f2);
        default:
            return s.stride == 1 ? launch_bits_cw8_s1(a32, w32, out, s, stream, thr, f2)
                                 : launch_bits_cw8_s2(a32, w32, out, s, stream, thr, f2);
    }
}

bool bconv_bn_residual_areg_supports(const ConvShape& s, const void* scale, const void* shift,
                                     const void* r, const void* x_out)
{
    // 16-byte loads of scale, shift and r, 16-byte stores of x_out, whole output words
    const uintptr_t bits = reinterpret_cast<uintptr_t>(scale) | reinterpret_cast<uintptr_t>(shift) |
                           reinterpret_cast<uintptr_t>(r) | reinterpret_cast<uintptr_t>(x_out);
    return bconv_bnsign_areg_supports(s) && r != nullptr && (bits & 15) == 0;
}

hipError_t launch_bconv_bn_residual_areg(const uint64_t* a, const uint64_t* w, const float* scale,
                                         const float* shift, const float* r, float* x_out,
                                         uint64_t* bits, const ConvShape& s, hipStream_t stream)
{
    if (!bconv_bn_residual_areg_supports(s, scale, shift, r, x_out))
        return hipErrorNotSupported;
    const uint32_t* a32 = reinterpret_cast<const uint32_t*>(a);
    const uint32_t* w32 = reinterpret_cast<const uint32_t*>(w);
#define DABNN_CASE(CW)                                                                             \
    return s.stride == 1 ? launch_res_cw##CW##_s1(a32, w32, s, stream, scale, shift, r, x_out, bits) \
                         : launch_res_cw##CW##_s2(a32, w32, s, stream, scale, shift, r, x_out, bits)
    switch (s.Cw) {
        case 1: DABNN_CASE(1);
        case 2: DABNN_CASE(2);
        case 4: DABNN_CASE(4);
        default: DABNN_CASE(8);
    }
#undef DABNN_CASE
}

bool bconv_areg_supports(const ConvShape& s, const void* y)
{
    if (!(s.kh == 3 && s.kw == 3 && (s.stride == 1 || s.stride == 2)))
        return false;
    if (!(s.Cw == 1 || s.Cw == 2 || s.Cw == 4 || s.Cw == 8))
        return false;
    const int cg = (s.Cw == 1) ? 8 : 4;
    return areg_offsets_fit(s) && s.Cout % cg == 0 && (reinterpret_cast<uintptr_t>(y) & 15) == 0;
}

hipError_t launch_bconv_areg(const uint64_t* a, const uint64_t* w, int32_t* y, const ConvShape& s,
                             hipStream_t stream)
{
    if (!bconv_areg_supports(s, y))
        return hipErrorNotSupported;
    const uint32_t* a32 = reinterpret_cast<const uint32_t*>(a);
    const uint32_t* w32 = reinterpret_cast<const uint32_t*>(w);
    switch (s.Cw) {
        case 1:
            return s.stride == 1 ? launch_areg_cw1_s1(a32, w32, y, s, stream)
                                 : launch_areg_cw1_s2(a32, w32, y, s, stream);
        case 2:
            return s.stride == 1 ? launch_areg_cw2_s1(a32, w32, y, s, stream)
                                 : launch_areg_cw2_s2(a32, w32, y, s, stream);
        case 4:
            return s.stride == 1 ? launch_areg_cw4_s1(a32, w32, y, s, stream)
                                 : launch_areg_cw4_s2(a32, w32, y, s, stream);
        default:
            return s.stride == 1 ? launch_areg_cw8_s1(a32, w32, y, s, stream)
                                 : launch_areg_cw8_s2(a32, w32, y, s, stream);
    }
}

}  // namespace dabnn

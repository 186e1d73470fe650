// Dispatch of the activation-stationary binary convolution family.  Kernels with one wavefront
// per channel group: bconv_areg_kernel.h, instantiated per word count and stride in
// bconv_areg_cw<Cw>_s<stride>.hip (up to 8 words per pixel).  Kernels in which the four wavefronts
// of a workgroup share a group: bconv_areg_split_kernel.h, instantiated in
// bconv_areg_split_cw<n>.hip (more than 8 words per pixel, as a few launches that add up).
#include "kernel_util.h"
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
#define DABNN_DECLARE_BOTH(CW) DABNN_DECLARE(CW, 1) DABNN_DECLARE(CW, 2)
DABNN_DECLARE_BOTH(1) DABNN_DECLARE_BOTH(2) DABNN_DECLARE_BOTH(3) DABNN_DECLARE_BOTH(4)
DABNN_DECLARE_BOTH(5) DABNN_DECLARE_BOTH(6) DABNN_DECLARE_BOTH(7) DABNN_DECLARE_BOTH(8)
#undef DABNN_DECLARE_BOTH
#undef DABNN_DECLARE
#define DABNN_DECLARE_SPLIT(C)                                                                     \
    hipError_t launch_split_cw##C(const uint32_t* a, const uint32_t* w, int32_t* y, int cw_total,  \
                                  int word0, bool first, int active_waves, const ConvShape& s,    \
                                  hipStream_t stream);
DABNN_DECLARE_SPLIT(1) DABNN_DECLARE_SPLIT(2) DABNN_DECLARE_SPLIT(3) DABNN_DECLARE_SPLIT(4)
#undef DABNN_DECLARE_SPLIT
hipError_t launch_split_bits_cw2(const uint32_t* a, const uint32_t* w, uint64_t* out,
                                 const int32_t* thr, const uint64_t* flip, const ConvShape& s,
                                 hipStream_t stream);

// The kernels address a window tap as the tensor base plus a 32-bit BYTE offset, and (on the
// direct-store path) the output with 32-bit element offsets: the packed activation tensor must
// stay below 4 GiB and the output below 2^31 elements.  The split kernels address the filters the
// same way (below 4 GiB).  Larger tensors run the other families, which index with size_t.
static bool areg_offsets_fit(const ConvShape& s)
{
    const int64_t act_bytes = static_cast<int64_t>(s.N) * s.H * s.W * s.Cw * 8;
    const int64_t out_elems = static_cast<int64_t>(s.N) * s.Ho * s.Wo * s.Cout;
    const int64_t filter_bytes = static_cast<int64_t>(s.Cout) * 72 * s.Cw;
    // (the transposed store addresses the 64 pixels of an output tile with a 32-bit byte offset)
    const int64_t out_tile_bytes = static_cast<int64_t>(s.Cout) * 64 * 4;
    return act_bytes < (int64_t{1} << 32) && out_elems < (int64_t{1} << 31) &&
           filter_bytes < (int64_t{1} << 32) && out_tile_bytes < (int64_t{1} << 32);
}

static bool areg_geometry(const ConvShape& s)
{
    return s.kh == 3 && s.kw == 3 && (s.stride == 1 || s.stride == 2) && areg_offsets_fit(s);
}

// Calls F(CW, S) for the shape's word count (1..8) and stride.
#define DABNN_SWITCH_CW_S(s, F)                                       \
    switch ((s).Cw * 2 + ((s).stride == 2 ? 1 : 0)) {                 \
        case 2: F(1, 1); case 3: F(1, 2); case 4: F(2, 1); case 5: F(2, 2);     \
        case 6: F(3, 1); case 7: F(3, 2); case 8: F(4, 1); case 9: F(4, 2);     \
        case 10: F(5, 1); case 11: F(5, 2); case 12: F(6, 1); case 13: F(6, 2); \
        case 14: F(7, 1); case 15: F(7, 2); case 16: F(8, 1); case 17: F(8, 2); \
        default: return hipErrorNotSupported;                         \
    }

// 8 words per pixel: the four-wavefront kernel or the one-wavefront kernel?
static bool use_split_at_8_words(const ConvShape& s)
{
    const int split_option = option(DABNN_OPT_AREG_SPLIT);
    if (s.Cout % 16 != 0 || option(DABNN_OPT_AREG_STORE) == 1 || split_option == 1)
        return false;
    // A latency-bound launch at 8 words (fewer than 3 groups per CU) is shorter with the
    // one-wavefront kernel's groups of 4 channels: 7x7x512->512 at batch 1 6.8 against 8.1 us, at
    // batch 24 11.7 against 13.9, at batch 32 13.7 against 13.0.
    const int64_t tiles = (static_cast<int64_t>(s.N) * s.Ho * s.Wo + 63) / 64;
    const bool few_groups = tiles * (s.Cout / 16) < 3 * static_cast<int64_t>(device_cu_count());
    return !few_groups || split_option == 8;
}

bool bconv_bnsign_areg_supports(const ConvShape& s)
{
    return areg_geometry(s) && s.Cw <= 8 && s.Cout % 64 == 0;
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
    // 8 words per pixel: the four-wavefront kernel, as for the plain convolution (7x7x512->512
    // at batch 256: 58 against 68 us), unless the launch is small or the option says otherwise
    if (s.Cw == 8 && use_split_at_8_words(s))
        return launch_split_bits_cw2(a32, w32, out, thr, flip, s, stream);
#define DABNN_CASE(CW, S) return launch_bits_cw##CW##_s##S(a32, w32, out, s, stream, thr, f2)
    DABNN_SWITCH_CW_S(s, DABNN_CASE)
#undef DABNN_CASE
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
#define DABNN_CASE(CW, S) return launch_res_cw##CW##_s##S(a32, w32, s, stream, scale, shift, r, x_out, bits)
    DABNN_SWITCH_CW_S(s, DABNN_CASE)
#undef DABNN_CASE
}

bool bconv_areg_small_launch(const ConvShape& s)
{
    // fewer than 2 (one word per pixel) or 2.5 sixteen-channel groups per SIMD
    const int64_t tiles = (static_cast<int64_t>(s.N) * s.Ho * s.Wo + 63) / 64;
    const int64_t simds = static_cast<int64_t>(device_cu_count()) * 4;
    return tiles * (s.Cout / 16) * 4 < simds * (s.Cw == 1 ? 8 : 10);
}

bool bconv_areg_supports(const ConvShape& s, const void* y)
{
    if (!areg_geometry(s) || (reinterpret_cast<uintptr_t>(y) & 15) != 0)
        return false;
    if (s.Cw > 8)
        return s.Cout % 16 == 0;   // the split kernels: several launches that add up
    // direct stores take 4 channels per group, 8 when the word count is odd
    return s.Cout % ((s.Cw % 2) ? 8 : 4) == 0;
}

hipError_t launch_bconv_areg(const uint64_t* a, const uint64_t* w, int32_t* y, const ConvShape& s,
                             hipStream_t stream)
{
    if (!bconv_areg_supports(s, y))
        return hipErrorNotSupported;
    const uint32_t* a32 = reinterpret_cast<const uint32_t*>(a);
    const uint32_t* w32 = reinterpret_cast<const uint32_t*>(w);
    // 8 words per pixel: the four-wavefront kernel is the faster one at batch 256 (55 against 57 us
    // per 59 G-op layer) and writes whole 64-byte runs where the one-wavefront kernel's direct
    // stores cost 2.25 times the output bytes in HBM writes, so it is the default there.
    // Option DABNN_OPT_AREG_SPLIT: 4 forces it for 4 words as well, 1 never uses it below 9 words.
    const int split_option = option(DABNN_OPT_AREG_SPLIT);
    const bool split_fits = s.Cw % 4 == 0 && s.Cout % 16 == 0 && option(DABNN_OPT_AREG_STORE) != 1;
    const bool use_split = s.Cw > 8 || (s.Cw == 8 && use_split_at_8_words(s)) ||
                           (split_fits && split_option == 4);
    if (!use_split) {
#define DABNN_CASE(CW, S) return launch_areg_cw##CW##_s##S(a32, w32, y, s, stream)
        DABNN_SWITCH_CW_S(s, DABNN_CASE)
#undef DABNN_CASE
    }
    // More than 8 words per pixel: the K dimension is covered by several four-wavefront launches
    // in a row, the first writing y = K - 2*P1, the others adding -2*Pi: 16, 12, 8 or 4 words at
    // a time, and a last one over the 1 to 3 words that remain, in which only that many
    // wavefronts of a workgroup have words to read.
    int word0 = 0;
    while (word0 < s.Cw) {
        const int left = s.Cw - word0;
        const int per_wave = left >= 16 ? 4 : (left >= 4 ? left / 4 : 1);
        const int active = left >= 4 ? 4 : left;
        const bool first = word0 == 0;
        hipError_t e;
        switch (per_wave) {
            case 1: e = launch_split_cw1(a32, w32, y, s.Cw, word0, first, active, s, stream); break;
            case 2: e = launch_split_cw2(a32, w32, y, s.Cw, word0, first, active, s, stream); break;
            case 3: e = launch_split_cw3(a32, w32, y, s.Cw, word0, first, active, s, stream); break;
            default: e = launch_split_cw4(a32, w32, y, s.Cw, word0, first, active, s, stream); break;
        }
        if (e != hipSuccess)
            return e;
        word0 += left >= 4 ? 4 * per_wave : left;
    }
    return hipSuccess;
}

}  // namespace dabnn

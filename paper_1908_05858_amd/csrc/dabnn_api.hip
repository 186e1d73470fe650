// C ABI of the library (see include/dabnn.h): argument validation, error codes, dispatch.
// Nothing here computes, with one host-side exception (dabnn_bn_thresholds, which turns batch-norm
// parameters into integer thresholds); every device step runs in the kernels of bitpack.hip,
// bconv*.hip and bgemm.hip.
#include "../../include/dabnn.h"

#include "launch.h"

#include "kernel_util.h"

#include <atomic>
#include <cmath>

namespace dabnn {

static std::atomic<int> g_options[DABNN_OPT_COUNT];  // zero-initialised: "the library chooses"

int option(int id)
{
    return g_options[id].load(std::memory_order_relaxed);
}

}  // namespace dabnn

namespace {

bool aligned(const void* p, uintptr_t a)
{
    return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0;
}

int out_dim(int in, int k, int stride, int pad)
{
    if (in <= 0 || k <= 0 || stride <= 0 || pad < 0 || pad >= k || in + 2 * pad < k)
        return -1;
    return (in + 2 * pad - k) / stride + 1;
}

constexpr int64_t kMaxElems = 0x7fffffffLL;  // every tensor is indexed with 32-bit element counts

int make_shape(dabnn::ConvShape& s, int N, int H, int W, int Cin, int Cout, int kh, int kw,
               int stride, int pad)
{
    if (N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || kh <= 0 || kw <= 0 || stride <= 0 ||
        pad < 0)
        return DABNN_ERR_SHAPE;
    if (pad >= kh || pad >= kw)
        return DABNN_ERR_SHAPE;
    const int Ho = out_dim(H, kh, stride, pad), Wo = out_dim(W, kw, stride, pad);
    if (Ho <= 0 || Wo <= 0)
        return DABNN_ERR_SHAPE;
    const int64_t Cw = (static_cast<int64_t>(Cin) + 63) / 64;
    const int64_t K = static_cast<int64_t>(kh) * kw * Cin;
    if (K >= (1LL << 30))
        return DABNN_ERR_SHAPE;
    if (static_cast<int64_t>(N) * H * W * Cw > kMaxElems ||
        static_cast<int64_t>(Cout) * kh * kw * Cw > kMaxElems ||
        static_cast<int64_t>(N) * Ho * Wo * Cout > kMaxElems)
        return DABNN_ERR_SHAPE;
    s = dabnn::ConvShape{N, H, W, Cin, Cout, kh, kw, stride, pad, Ho, Wo, static_cast<int>(Cw),
                         static_cast<int>(K)};
    return DABNN_OK;
}

// A 1x1, stride-1, unpadded convolution is the BGEMM of the [N*H*W][Cw] activation matrix with the
// [Cout][Cw] filter matrix.
bool conv_is_gemm(const dabnn::ConvShape& s)
{
    return s.kh == 1 && s.kw == 1 && s.stride == 1 && s.pad == 0;
}

int pick_algo(const dabnn::ConvShape& s, const void* y)
{
    // Measured on MI355X at the Bi-Real-18 shapes, the activation-stationary family is the
    // faster one wherever it applies; the filter-stationary family covers Cout % 4 != 0.
    if (dabnn::bconv_areg_supports(s, y))
        return DABNN_ALGO_AREG;
    if (conv_is_gemm(s) &&
        dabnn::bgemm_rowreg_supports(static_cast<int64_t>(s.N) * s.H * s.W, s.Cout, s.Cw, y))
        return DABNN_ALGO_BGEMM;
    if (dabnn::bconv_wreg_supports(s))
        return DABNN_ALGO_WREG;
    return DABNN_ALGO_REFERENCE;
}

}  // namespace

extern "C" {

int dabnn_set_option(int option, int value)
{
    if (option < 0 || option >= DABNN_OPT_COUNT || value < 0)
        return DABNN_ERR_UNSUPPORTED;
    dabnn::g_options[option].store(value, std::memory_order_relaxed);
    return DABNN_OK;
}

int dabnn_get_option(int option)
{
    if (option < 0 || option >= DABNN_OPT_COUNT)
        return -1;
    return dabnn::option(option);
}

int64_t dabnn_packed_words(int64_t C)
{
    return C <= 0 ? -1 : (C + 63) / 64;
}

int dabnn_conv_out_dim(int in, int k, int stride, int pad)
{
    return out_dim(in, k, stride, pad);
}

int dabnn_bitpack(const float* x, uint64_t* out, int64_t n_pixels, int C, int sign_mode,
                  void* stream)
{
    if (n_pixels < 0 || C <= 0 || n_pixels > (1LL << 40) / C)
        return DABNN_ERR_SHAPE;
    if (n_pixels == 0)
        return DABNN_OK;  // nothing to do; empty tensors may have NULL storage
    if (!x || !out)
        return DABNN_ERR_NULL;
    if (!aligned(x, 4) || !aligned(out, 8))
        return DABNN_ERR_ALIGN;
    if (sign_mode != DABNN_SIGN_BIT && sign_mode != DABNN_SIGN_GE0)
        return DABNN_ERR_UNSUPPORTED;
    const hipError_t e =
        dabnn::launch_bitpack(x, out, n_pixels, C, sign_mode, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? DABNN_OK : DABNN_ERR_LAUNCH;
}

int dabnn_bitpack_i32(const int32_t* x, uint64_t* out, int64_t n_pixels, int C, void* stream)
{
    // The sign bit of an int32 is bit 31, like that of an fp32: the same kernel on the raw bits.
    return dabnn_bitpack(reinterpret_cast<const float*>(x), out, n_pixels, C, DABNN_SIGN_BIT, stream);
}

static int layout_call(const uint64_t* in, uint64_t* out, int N, int H, int W, int Cw, bool to_grouped,
                       void* stream)
{
    if (!in || !out)
        return DABNN_ERR_NULL;
    if (N <= 0 || H <= 0 || W <= 0 || Cw <= 0 ||
        static_cast<int64_t>(N) * H * W * (Cw + 1) > kMaxElems)
        return DABNN_ERR_SHAPE;
    if (!aligned(in, 8) || !aligned(out, 8))
        return DABNN_ERR_ALIGN;
    const hipError_t e =
        dabnn::launch_nc1hwc2(in, out, N, H, W, Cw, to_grouped, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? DABNN_OK : DABNN_ERR_LAUNCH;
}

int dabnn_nhwc_to_nc1hwc2(const uint64_t* in, uint64_t* out, int N, int H, int W, int Cw, void* stream)
{
    return layout_call(in, out, N, H, W, Cw, true, stream);
}

int dabnn_nc1hwc2_to_nhwc(const uint64_t* in, uint64_t* out, int N, int H, int W, int Cw, void* stream)
{
    return layout_call(in, out, N, H, W, Cw, false, stream);
}

int dabnn_bn_sign_pack(const int32_t* y, const float* scale, const float* shift, const float* r,
                       float* x_out, uint64_t* bits, int64_t n_pixels, int C, void* stream)
{
    if (n_pixels < 0 || C <= 0 || n_pixels > (1LL << 40) / C)
        return DABNN_ERR_SHAPE;
    if (n_pixels == 0)
        return DABNN_OK;
    if (!y || !scale || !shift || !bits)
        return DABNN_ERR_NULL;
    if (!aligned(y, 4) || !aligned(scale, 4) || !aligned(shift, 4) || !aligned(r, 4) ||
        !aligned(x_out, 4) || !aligned(bits, 8))
        return DABNN_ERR_ALIGN;
    const hipError_t e = dabnn::launch_bn_sign_pack(y, scale, shift, r, x_out, bits, n_pixels, C,
                                                    static_cast<hipStream_t>(stream));
    return e == hipSuccess ? DABNN_OK : DABNN_ERR_LAUNCH;
}

int dabnn_pack_weights(const float* w, uint64_t* out, int Cout, int kh, int kw, int Cin,
                       int sign_mode, void* stream)
{
    if (!w || !out)
        return DABNN_ERR_NULL;
    if (Cout <= 0 || kh <= 0 || kw <= 0 || Cin <= 0)
        return DABNN_ERR_SHAPE;
    const int64_t rows = static_cast<int64_t>(Cout) * kh * kw;
    if (rows > kMaxElems || rows * Cin > kMaxElems)
        return DABNN_ERR_SHAPE;
    if (!aligned(w, 4) || !aligned(out, 8))
        return DABNN_ERR_ALIGN;
    if (sign_mode != DABNN_SIGN_BIT && sign_mode != DABNN_SIGN_GE0)
        return DABNN_ERR_UNSUPPORTED;
    // A filter tap is one "pixel" of Cin channels: the canonical layout is the packer's output.
    const hipError_t e =
        dabnn::launch_bitpack(w, out, rows, Cin, sign_mode, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? DABNN_OK : DABNN_ERR_LAUNCH;
}

int dabnn_bconv2d_algo(const uint64_t* a, const uint64_t* w, int32_t* y, int N, int H, int W,
                       int Cin, int Cout, int kh, int kw, int stride, int pad, int algo,
                       void* stream)
{
    if (!a || !w || !y)
        return DABNN_ERR_NULL;
    dabnn::ConvShape s;
    const int rc = make_shape(s, N, H, W, Cin, Cout, kh, kw, stride, pad);
    if (rc != DABNN_OK)
        return rc;
    if (!aligned(a, 8) || !aligned(w, 8) || !aligned(y, 4))
        return DABNN_ERR_ALIGN;
    if (algo == DABNN_ALGO_AUTO)
        algo = pick_algo(s, y);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e;
    switch (algo) {
        case DABNN_ALGO_REFERENCE: e = dabnn::launch_bconv_reference(a, w, y, s, st); break;
        case DABNN_ALGO_WREG: e = dabnn::launch_bconv_wreg(a, w, y, s, st); break;
        case DABNN_ALGO_AREG: e = dabnn::launch_bconv_areg(a, w, y, s, st); break;
        case DABNN_ALGO_BGEMM:
            e = conv_is_gemm(s) ? dabnn::launch_bgemm_rowreg(a, w, y, static_cast<int64_t>(s.N) * s.H * s.W,
                                                             s.Cout, s.Cw, s.K, DABNN_BGEMM_SIGNED, st)
                                : hipErrorNotSupported;
            break;
        default: return DABNN_ERR_UNSUPPORTED;
    }
    if (e == hipErrorNotSupported)
        return DABNN_ERR_UNSUPPORTED;
    return e == hipSuccess ? DABNN_OK : DABNN_ERR_LAUNCH;
}

int dabnn_bconv2d(const uint64_t* a, const uint64_t* w, int32_t* y, int N, int H, int W, int Cin,
                  int Cout, int kh, int kw, int stride, int pad, void* stream)
{
    return dabnn_bconv2d_algo(a, w, y, N, H, W, Cin, Cout, kh, kw, stride, pad, DABNN_ALGO_AUTO,
                              stream);
}

int dabnn_bgemm(const uint64_t* A, const uint64_t* B, int32_t* C, int64_t M, int N, int Kw, int K,
                int mode, void* stream)
{
    if (!A || !B || !C)
        return DABNN_ERR_NULL;
    if (M <= 0 || N <= 0 || Kw <= 0 || K <= 0 || K > 64LL * Kw || K >= (1 << 23))
        return DABNN_ERR_SHAPE;
    if (M * Kw > kMaxElems || static_cast<int64_t>(N) * Kw > kMaxElems || M * N > kMaxElems)
        return DABNN_ERR_SHAPE;
    if (!aligned(A, 8) || !aligned(B, 8) || !aligned(C, 4))
        return DABNN_ERR_ALIGN;
    if (mode != DABNN_BGEMM_SIGNED && mode != DABNN_BGEMM_MATCHES)
        return DABNN_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const hipError_t e = dabnn::bgemm_rowreg_supports(M, N, Kw, C)
                             ? dabnn::launch_bgemm_rowreg(A, B, C, M, N, Kw, K, mode, st)
                             : dabnn::launch_bgemm_reference(A, B, C, M, N, Kw, K, mode, st);
    return e == hipSuccess ? DABNN_OK : DABNN_ERR_LAUNCH;
}

int dabnn_im2col(const uint64_t* a, uint64_t* cols, int N, int H, int W, int Cin, int kh, int kw,
                 int stride, int pad, void* stream)
{
    if (!a || !cols)
        return DABNN_ERR_NULL;
    dabnn::ConvShape s;
    const int rc = make_shape(s, N, H, W, Cin, 1, kh, kw, stride, pad);
    if (rc != DABNN_OK)
        return rc;
    if (static_cast<int64_t>(N) * s.Ho * s.Wo * kh * kw * s.Cw > kMaxElems)
        return DABNN_ERR_SHAPE;
    if (!aligned(a, 8) || !aligned(cols, 8))
        return DABNN_ERR_ALIGN;
    const hipError_t e = dabnn::launch_im2col(a, cols, s, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? DABNN_OK : DABNN_ERR_LAUNCH;
}

int dabnn_expand_int8(const uint64_t* bits, int8_t* out, int64_t rows, int C, void* stream)
{
    if (rows < 0 || C <= 0 || rows > (1LL << 40) / C)
        return DABNN_ERR_SHAPE;
    if (rows == 0)
        return DABNN_OK;
    if (!bits || !out)
        return DABNN_ERR_NULL;
    if (!aligned(bits, 8) || !aligned(out, 16))
        return DABNN_ERR_ALIGN;
    if (C % 64 != 0)
        return DABNN_ERR_UNSUPPORTED;
    const hipError_t e = dabnn::launch_expand_pm1(bits, out, rows, C, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? DABNN_OK : DABNN_ERR_LAUNCH;
}

int dabnn_bconv2d_int8(const int8_t* a8, const int8_t* w8, int32_t* y, int N, int H, int W, int Cin,
                       int Cout, int kh, int kw, int stride, int pad, void* stream)
{
    if (!a8 || !w8 || !y)
        return DABNN_ERR_NULL;
    dabnn::ConvShape s;
    const int rc = make_shape(s, N, H, W, Cin, Cout, kh, kw, stride, pad);
    if (rc != DABNN_OK)
        return rc;
    if (static_cast<int64_t>(N) * H * W * Cin > kMaxElems ||
        static_cast<int64_t>(Cout) * kh * kw * Cin > kMaxElems)
        return DABNN_ERR_SHAPE;
    if (!aligned(a8, 16) || !aligned(w8, 16) || !aligned(y, 4))
        return DABNN_ERR_ALIGN;
    if (!dabnn::bconv_mfma_supports(s))
        return DABNN_ERR_UNSUPPORTED;
    const hipError_t e = dabnn::launch_bconv_mfma_i8(a8, w8, y, s, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? DABNN_OK : DABNN_ERR_LAUNCH;
}

static bool mfma_format_ok(int format)
{
    return format == DABNN_MFMA_INT8 || format == DABNN_MFMA_FP4;
}

size_t dabnn_mfma_weights_bytes(int Cin, int Cout, int kh, int kw, int format)
{
    dabnn::ConvShape s;
    if (!mfma_format_ok(format) || make_shape(s, 1, kh, kw, Cin, Cout, kh, kw, 1, 0) != DABNN_OK ||
        !dabnn::bconv_mfma_bits_supports(s))
        return 0;
    return dabnn::mfma_weights_bytes(s, format);
}

int dabnn_prepare_weights_mfma(const uint64_t* w, void* wq, int Cin, int Cout, int kh, int kw,
                               int format, void* stream)
{
    if (!w || !wq)
        return DABNN_ERR_NULL;
    dabnn::ConvShape s;
    const int rc = make_shape(s, 1, kh, kw, Cin, Cout, kh, kw, 1, 0);
    if (rc != DABNN_OK)
        return rc;
    if (!aligned(w, 8) || !aligned(wq, 16))
        return DABNN_ERR_ALIGN;
    if (!dabnn::bconv_mfma_bits_supports(s) || !mfma_format_ok(format))
        return DABNN_ERR_UNSUPPORTED;
    const hipError_t e = dabnn::launch_prepare_weights_mfma(w, wq, s, format, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? DABNN_OK : DABNN_ERR_LAUNCH;
}

int dabnn_bconv2d_mfma(const uint64_t* a, const void* wq, int32_t* y, int N, int H, int W, int Cin,
                       int Cout, int kh, int kw, int stride, int pad, int format, void* stream)
{
    if (!a || !wq || !y)
        return DABNN_ERR_NULL;
    dabnn::ConvShape s;
    const int rc = make_shape(s, N, H, W, Cin, Cout, kh, kw, stride, pad);
    if (rc != DABNN_OK)
        return rc;
    if (!aligned(a, 16) || !aligned(wq, 16) || !aligned(y, 4))
        return DABNN_ERR_ALIGN;
    if (!dabnn::bconv_mfma_bits_supports(s) || !mfma_format_ok(format))
        return DABNN_ERR_UNSUPPORTED;
    const hipError_t e = dabnn::launch_bconv_mfma_bits(a, wq, y, nullptr, nullptr, s, format,
                                                       static_cast<hipStream_t>(stream));
    return e == hipSuccess ? DABNN_OK : DABNN_ERR_LAUNCH;
}

int dabnn_bconv2d_bnsign_mfma(const uint64_t* a, const void* wq, const int32_t* thr,
                              const uint64_t* flip, uint64_t* out, int N, int H, int W, int Cin,
                              int Cout, int kh, int kw, int stride, int pad, int format, void* stream)
{
    if (!a || !wq || !thr || !flip || !out)
        return DABNN_ERR_NULL;
    dabnn::ConvShape s;
    const int rc = make_shape(s, N, H, W, Cin, Cout, kh, kw, stride, pad);
    if (rc != DABNN_OK)
        return rc;
    if (!aligned(a, 16) || !aligned(wq, 16) || !aligned(thr, 4) || !aligned(flip, 8) || !aligned(out, 8))
        return DABNN_ERR_ALIGN;
    if (!dabnn::bconv_mfma_bits_supports(s) || !mfma_format_ok(format))
        return DABNN_ERR_UNSUPPORTED;
    const hipError_t e = dabnn::launch_bconv_mfma_bits(a, wq, reinterpret_cast<int32_t*>(out), thr, flip, s,
                                                       format, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? DABNN_OK : DABNN_ERR_LAUNCH;
}

int dabnn_bconv2d_zeropad(const uint64_t* a, const uint64_t* w, int32_t* y, int N, int H, int W,
                          int Cin, int Cout, int kh, int kw, int stride, int pad, void* stream)
{
    const int rc = dabnn_bconv2d_algo(a, w, y, N, H, W, Cin, Cout, kh, kw, stride, pad,
                                      DABNN_ALGO_AUTO, stream);
    if (rc != DABNN_OK || pad == 0)
        return rc;
    dabnn::ConvShape s;
    make_shape(s, N, H, W, Cin, Cout, kh, kw, stride, pad);  // validated by the call above
    const hipError_t e = dabnn::launch_bconv_zeropad_fix(w, y, s, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? DABNN_OK : DABNN_ERR_LAUNCH;
}

int dabnn_bconv2d_bnsign(const uint64_t* a, const uint64_t* w, const int32_t* thr,
                         const uint64_t* flip, uint64_t* out, int N, int H, int W, int Cin,
                         int Cout, int kh, int kw, int stride, int pad, void* stream)
{
    if (!a || !w || !thr || !flip || !out)
        return DABNN_ERR_NULL;
    dabnn::ConvShape s;
    const int rc = make_shape(s, N, H, W, Cin, Cout, kh, kw, stride, pad);
    if (rc != DABNN_OK)
        return rc;
    if (!aligned(a, 8) || !aligned(w, 8) || !aligned(thr, 4) || !aligned(flip, 8) || !aligned(out, 8))
        return DABNN_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const hipError_t e = dabnn::bconv_bnsign_areg_supports(s)
                             ? dabnn::launch_bconv_bnsign_areg(a, w, thr, flip, out, s, st)
                             : dabnn::launch_bconv_bnsign_reference(a, w, thr, flip, out, s, st);
    return e == hipSuccess ? DABNN_OK : DABNN_ERR_LAUNCH;
}

int dabnn_bconv2d_bn_residual(const uint64_t* a, const uint64_t* w, const float* scale,
                              const float* shift, const float* r, float* x_out, uint64_t* bits,
                              int N, int H, int W, int Cin, int Cout, int kh, int kw, int stride,
                              int pad, void* stream)
{
    if (!a || !w || !scale || !shift || !x_out || !bits)
        return DABNN_ERR_NULL;
    dabnn::ConvShape s;
    const int rc = make_shape(s, N, H, W, Cin, Cout, kh, kw, stride, pad);
    if (rc != DABNN_OK)
        return rc;
    if (!aligned(a, 8) || !aligned(w, 8) || !aligned(scale, 4) || !aligned(shift, 4) ||
        !aligned(r, 4) || !aligned(x_out, 4) || !aligned(bits, 8))
        return DABNN_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // The one-kernel route works in 16- or 32-channel groups.  A small launch (a single image, a
    // small batch) is bound by the latency of those groups; the convolution with its short
    // direct-store groups followed by the layer kernel is faster there (one image through the 16
    // Bi-Real-18 blocks: 100 against 142 us of device time; level at batch 16).
    const int route = dabnn::option(DABNN_OPT_RES_FUSED);   // 0 by size, 1 one kernel, 2 two kernels
    const bool one_kernel = route == 1 || (route == 0 && !dabnn::bconv_areg_small_launch(s));
    if (one_kernel && dabnn::bconv_bn_residual_areg_supports(s, scale, shift, r, x_out)) {
        const hipError_t e =
            dabnn::launch_bconv_bn_residual_areg(a, w, scale, shift, r, x_out, bits, s, st);
        return e == hipSuccess ? DABNN_OK : DABNN_ERR_LAUNCH;
    }
    // Any other shape: the convolution writes its int32 result into x_out's storage (same size),
    // and the layer kernel turns every element into z in place (each thread reads y[e] before it
    // writes z[e]).
    int32_t* y = reinterpret_cast<int32_t*>(x_out);
    const int rc2 = dabnn_bconv2d(a, w, y, N, H, W, Cin, Cout, kh, kw, stride, pad, stream);
    if (rc2 != DABNN_OK)
        return rc2;
    const hipError_t e = dabnn::launch_bn_sign_pack(y, scale, shift, r, x_out, bits,
                                                    static_cast<int64_t>(N) * s.Ho * s.Wo, Cout, st);
    return e == hipSuccess ? DABNN_OK : DABNN_ERR_LAUNCH;
}

int dabnn_bn_thresholds(const float* gamma, const float* beta, const float* mean, const float* var,
                        float eps, int Cout, int K, int32_t* thr, uint64_t* flip)
{
    if (!gamma || !beta || !mean || !var || !thr || !flip)
        return DABNN_ERR_NULL;
    if (Cout <= 0 || K <= 0 || K >= (1 << 30))
        return DABNN_ERR_SHAPE;
    for (int j = 0; j < (Cout + 63) / 64; ++j)
        flip[j] = 0;
    for (int c = 0; c < Cout; ++c) {
        const double g = gamma[c], b = beta[c], m = mean[c];
        const double sd = std::sqrt(static_cast<double>(var[c]) + static_cast<double>(eps));
        // the batch-norm output for the integer conv value y, in the order the layer is defined
        auto negative = [&](int y) { return g * (static_cast<double>(y) - m) / sd + b < 0.0; };
        // z is monotone in y (rounding keeps monotonicity), so the set {y : z < 0} is a prefix
        // (gamma > 0), a suffix (gamma < 0) or all/nothing: find the boundary by bisection.
        const bool lo_neg = negative(-K), hi_neg = negative(K);
        int t;
        bool fl;
        if (lo_neg == hi_neg) {  // constant on [-K, K] (also gamma == 0 and NaN parameters)
            t = -K;              // y < -K never holds
            fl = lo_neg;
        } else {
            int lo = -K, hi = K;  // negative(lo) != negative(hi): the answer flips in (lo, hi]
            while (hi - lo > 1) {
                const int mid = lo + (hi - lo) / 2;
                if (negative(mid) == lo_neg)
                    lo = mid;
                else
                    hi = mid;
            }
            t = hi;               // first y where the sign differs from the one at -K
            fl = !lo_neg;         // prefix negative: bit = y < t; suffix negative: bit = !(y < t)
        }
        thr[c] = t;
        if (fl)
            flip[c / 64] |= 1ull << (c % 64);
    }
    return DABNN_OK;
}

int dabnn_bconv2d_pick_algo(int N, int H, int W, int Cin, int Cout, int kh, int kw, int stride,
                            int pad)
{
    dabnn::ConvShape s;
    if (make_shape(s, N, H, W, Cin, Cout, kh, kw, stride, pad) != DABNN_OK)
        return -1;
    return pick_algo(s, nullptr);
}

const char* dabnn_status_string(int status)
{
    switch (status) {
        case DABNN_OK: return "ok";
        case DABNN_ERR_NULL: return "null pointer";
        case DABNN_ERR_SHAPE: return "invalid shape";
        case DABNN_ERR_ALIGN: return "misaligned pointer";
        case DABNN_ERR_UNSUPPORTED: return "unsupported mode, algorithm or shape";
        case DABNN_ERR_LAUNCH: return "kernel launch failed";
        default: return "unknown status";
    }
}

}  // extern "C"

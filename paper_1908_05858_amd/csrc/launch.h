// Internal launch interface between the C ABI (dabnn_api.hip) and the kernel files.
// Arguments are already validated when these are called.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dabnn {

struct ConvShape {
    int N, H, W, Cin, Cout, kh, kw, stride, pad;
    int Ho, Wo, Cw;   // derived: output extent, 64-bit words per pixel
    int K;            // kh*kw*Cin, true bit count under one output
};

// Sign + pack rows of C fp32 values into ceil(C/64) words each (Sec. 2.1.1).
hipError_t launch_bitpack(const float* x, uint64_t* out, int64_t n_rows, int C, int sign_mode,
                          hipStream_t stream);

// Fused BN + shortcut + sign + pack (Sec. 2.1.1 / 2.3): z = ((scale*y) + shift) + r in fp32 without
// FMA, z -> x_out (optional), sign bits of z -> bits.  r and x_out may be null.
hipError_t launch_bn_sign_pack(const int32_t* y, const float* scale, const float* shift,
                               const float* r, float* x_out, uint64_t* bits, int64_t n_rows, int C,
                               hipStream_t stream);

// Packed NHWC [N][H][W][Cw] <-> NC1HWC2 [N][ceil(Cw/2)][H][W][2] (Sec. 2.1.2, C2 = 128 bits).
hipError_t launch_nc1hwc2(const uint64_t* in, uint64_t* out, int N, int H, int W, int Cw,
                          bool to_grouped, hipStream_t stream);

// Binary convolution kernels (Sec. 2.1.2, Eq. 6-7).  Each returns hipErrorNotSupported, without
// launching, when the family cannot run the shape.
hipError_t launch_bconv_reference(const uint64_t* a, const uint64_t* w, int32_t* y,
                                  const ConvShape& s, hipStream_t stream);
hipError_t launch_bconv_wreg(const uint64_t* a, const uint64_t* w, int32_t* y,
                             const ConvShape& s, hipStream_t stream);
hipError_t launch_bconv_areg(const uint64_t* a, const uint64_t* w, int32_t* y,
                             const ConvShape& s, hipStream_t stream);
// Fused conv + threshold + bit-pack (Sec. 2.1.1, fused BN-binarization): tuned and reference.
hipError_t launch_bconv_bnsign_areg(const uint64_t* a, const uint64_t* w, const int32_t* thr,
                                    const uint64_t* flip, uint64_t* out, const ConvShape& s,
                                    hipStream_t stream);
hipError_t launch_bconv_bnsign_reference(const uint64_t* a, const uint64_t* w, const int32_t* thr,
                                         const uint64_t* flip, uint64_t* out, const ConvShape& s,
                                         hipStream_t stream);
// In-place correction of a finished +1-padded convolution output to zero padding (border pixels
// only).  Any shape.
hipError_t launch_bconv_zeropad_fix(const uint64_t* w, int32_t* y, const ConvShape& s,
                                    hipStream_t stream);
// BGEMM (Sec. 2.1.2, Eq. 1) on packed row-major A [M][Kw], B [N][Kw] -> C [M][N]; mode 0: +-1 dot
// product K - 2*popcount(xor), mode 1: match count K - popcount(xor).
hipError_t launch_bgemm_rowreg(const uint64_t* A, const uint64_t* B, int32_t* C, int64_t M, int N,
                               int Kw, int K, int mode, hipStream_t stream);
hipError_t launch_bgemm_reference(const uint64_t* A, const uint64_t* B, int32_t* C, int64_t M, int N,
                                  int Kw, int K, int mode, hipStream_t stream);
bool bgemm_rowreg_supports(int64_t M, int N, int Kw, const void* C);
// Patch matrix [N*Ho*Wo][kh*kw][Cw] of a packed NHWC tensor (outside taps = zero words).
hipError_t launch_im2col(const uint64_t* a, uint64_t* cols, const ConvShape& s, hipStream_t stream);
// Expanded-operand comparison route: bits -> +-1 int8, and an int8 matrix-core implicit GEMM.
hipError_t launch_expand_pm1(const uint64_t* bits, int8_t* out, int64_t rows, int C,
                             hipStream_t stream);
hipError_t launch_bconv_mfma_i8(const int8_t* a8, const int8_t* w8, int32_t* y, const ConvShape& s,
                                hipStream_t stream);
bool bconv_mfma_supports(const ConvShape& s);
// Matrix-core route fed from the packed activation bits; filters prepared once per model.
bool bconv_mfma_bits_supports(const ConvShape& s);
// format 0: int8 operands, 1: FP4 (E2M1) operands.
size_t mfma_weights_bytes(const ConvShape& s, int format);
hipError_t launch_prepare_weights_mfma(const uint64_t* w, void* wq, const ConvShape& s, int format,
                                       hipStream_t stream);
// thr == nullptr: y is the int32 output; otherwise y is the packed output of the fused threshold
// epilogue (u64 [N][Ho][Wo][Cout/64]), bit c = (conv < thr[c]) XOR bit c of flip.
hipError_t launch_bconv_mfma_bits(const uint64_t* a, const void* wq, int32_t* y, const int32_t* thr,
                                  const uint64_t* flip, const ConvShape& s, int format,
                                  hipStream_t stream);
// Convolution with the BN + shortcut + sign + pack layer fused into its epilogue (no int32 tensor).
hipError_t launch_bconv_bn_residual_areg(const uint64_t* a, const uint64_t* w, const float* scale,
                                         const float* shift, const float* r, float* x_out,
                                         uint64_t* bits, const ConvShape& s, hipStream_t stream);
bool bconv_bn_residual_areg_supports(const ConvShape& s, const void* scale, const void* shift,
                                     const void* r, const void* x_out);
bool bconv_bnsign_areg_supports(const ConvShape& s);
bool bconv_wreg_supports(const ConvShape& s);
bool bconv_areg_supports(const ConvShape& s, const void* y);
// A launch with only a few 16-channel groups per SIMD (a single image, a small batch): bound by the
// latency of its groups, not by throughput.
bool bconv_areg_small_launch(const ConvShape& s);

}  // namespace dabnn

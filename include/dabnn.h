/*
 * dabnn.h -- C ABI of the MI355X (gfx950) bit-packing + binary direct convolution library.
 *
 * The operations are the two binary operators of daBNN (arXiv 1908.05858): bit-packing of the
 * sign of fp32 tensors (Sec. 2.1.1) and binary convolution computed as popcounts of XORed
 * bit-vectors (Sec. 2.1.2, Eq. 1 and Eq. 6-7), with weights packed ahead of time (Sec. 3).
 *
 * Conventions common to every call
 *   - Every tensor pointer is a DEVICE pointer owned by the caller.  The library never
 *     allocates, frees, copies to the host or synchronises.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  A call validates
 *     its arguments on the host, enqueues its kernel(s) on `stream` and returns at once.
 *   - Return value: a dabnn_status (0 = DABNN_OK).  An argument error (status 1-4) is found on
 *     the host before anything is launched: no output byte is written.  DABNN_ERR_LAUNCH means
 *     the HIP runtime refused a launch; the calls that enqueue two kernels
 *     (dabnn_bconv2d_zeropad with pad > 0, and dabnn_bconv2d_bn_residual on shapes outside its
 *     fused kernel) may then already have enqueued the first, so their outputs are undefined.
 *     No exception crosses the boundary.
 *   - The first call that reaches a given kernel asks the HIP runtime once for that kernel's
 *     occupancy (hipOccupancyMaxActiveBlocksPerMultiprocessor) and the device's CU count; the
 *     answers are cached for the life of the process.  Under stream capture, call each entry
 *     point once eagerly beforehand.
 *   - The library reads no environment variable.  dabnn_set_option is the only switch.
 *   - Tensors are dense, row-major, in the layouts stated per call.  Input and output buffers
 *     of one call must not overlap.
 *   - Bit convention (shared by activations and weights): bit 1 <-> value -1, bit 0 <-> +1;
 *     channel c lives in 64-bit word c/64 at bit c%64 (least significant bit first); bits past
 *     the last channel of a pixel are 0.
 */
#ifndef DABNN_H
#define DABNN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DABNN_OK = 0,
    DABNN_ERR_NULL = 1,        /* a required pointer is NULL */
    DABNN_ERR_SHAPE = 2,       /* a size is <= 0, inconsistent, or too large for int32 indexing */
    DABNN_ERR_ALIGN = 3,       /* fp32/int32 buffer not 4-byte or packed buffer not 8-byte aligned */
    DABNN_ERR_UNSUPPORTED = 4, /* unknown sign_mode / algo, or algo cannot run this shape */
    DABNN_ERR_LAUNCH = 5       /* the HIP runtime refused the launch */
} dabnn_status;

typedef enum {
    DABNN_SIGN_BIT = 0, /* Sec. 2.1.1: the bit is the IEEE-754 sign bit (-0.0 -> -1, NaN by its sign) */
    DABNN_SIGN_GE0 = 1  /* the bit is !(x >= 0): -0.0 -> +1, every NaN -> -1 */
} dabnn_sign_mode;

typedef enum {
    DABNN_ALGO_AUTO = 0,      /* fastest kernel that supports the shape */
    DABNN_ALGO_REFERENCE = 1, /* one thread per output, any shape; the GPU-side safety net */
    DABNN_ALGO_WREG = 2,      /* weights resident in VGPRs, activations broadcast through SGPRs;
                                 3x3 kernels with ceil(Cin/64) in {1,2,4,8}, stride 1 or 2 */
    DABNN_ALGO_AREG = 3,      /* each lane keeps one output pixel's 3x3 window (or, from 8 words per pixel
                                 on, a quarter of it) in VGPRs, weights are broadcast through SGPRs; 3x3
                                 kernels, stride 1 or 2, any Cin; Cout % 4 == 0 (% 8 for an odd number of
                                 words per pixel, % 16 above 8 words), y 16-byte aligned, packed
                                 activations and packed filters below 4 GiB, the output below 2^31
                                 elements, Cout below 2^24 */
    DABNN_ALGO_BGEMM = 4      /* 1x1, stride 1, pad 0 only: the convolution IS the BGEMM of Eq. 1;
                                 Cout % 16 == 0 and below 2^24, y 16-byte aligned, packed activations
                                 below 4 GiB, row lengths dabnn_bgemm's fast kernel supports */
} dabnn_algo;

typedef enum {
    DABNN_BGEMM_SIGNED = 0,  /* sum_k A_ik * B_jk over +-1 values = 2*C_ij - K (what the convolutions return) */
    DABNN_BGEMM_MATCHES = 1  /* C_ij of Eq. 1 as printed: bitcount(xnor), the number of agreeing bits */
} dabnn_bgemm_mode;

/*
 * Tuning and test options.  Every option is 0 by default, which means "the library chooses";
 * production code has no reason to set any.  They exist so that tests can reach every kernel
 * variant and every work split on any shape.  Values are process-wide, read at each call with
 * relaxed atomic loads; setting one while another thread is inside a call affects either that
 * call or the next.
 */
typedef enum {
    DABNN_OPT_AREG_SLOTS = 0,      /* n > 0: cut the work of a DABNN_ALGO_AREG launch into n ranges (wavefronts) */
    DABNN_OPT_AREG_TAIL = 1,       /* uneven remainder of that split handed out as small pieces: 1 never, 2 always */
    DABNN_OPT_AREG_STORE = 2,      /* output store of DABNN_ALGO_AREG: 1 direct 16-byte stores, 16 channels
                                      transposed through LDS (ignored if Cout is no multiple of 16) */
    DABNN_OPT_RES_CHANNELS = 3,    /* 16: 16-channel groups in dabnn_bconv2d_bn_residual's fused kernel */
    DABNN_OPT_WREG_PIXELS = 4,     /* 7 or 8: output pixels per task of DABNN_ALGO_WREG */
    DABNN_OPT_BGEMM_COLUMNS = 5,   /* 16: 16-column groups in dabnn_bgemm's fast kernel */
    DABNN_OPT_BITPACK_ROWWISE = 6, /* channel counts that are no multiple of 64: 1 the row-wise kernel, 2 the
                                      flat-stream kernel with 64-bit indices (by default only from 2^31 elements) */
    DABNN_OPT_AREG_SPLIT = 7,      /* DABNN_ALGO_AREG kernels in which the four wavefronts of a workgroup share a
                                      channel group (always used above 8 words per pixel, by default at 8 when
                                      Cout % 16 == 0 and the launch has 3 or more groups per CU): 1 not below 9
                                      words, 4 also at 4 words, 8 at 8 words whatever the launch's size */
    DABNN_OPT_AREG_RANGES_PER_SIMD = 8, /* n > 0: cut the work of a DABNN_ALGO_AREG launch into n ranges per SIMD */
    DABNN_OPT_MFMA_PIXEL_BLOCKS = 9, /* dabnn_bconv2d_mfma: 2 or 4 blocks of 32 pixels per wavefront */
    DABNN_OPT_RES_FUSED = 10,      /* dabnn_bconv2d_bn_residual: 1 the one-kernel route wherever it applies (by
                                      default not for small launches), 2 always convolution + layer kernel */
    DABNN_OPT_COUNT = 11
} dabnn_option;

/* Sets option `option` (a dabnn_option) to `value` and returns DABNN_OK, or DABNN_ERR_UNSUPPORTED
 * for an unknown option or a negative value.  dabnn_get_option returns the current value, or -1. */
int dabnn_set_option(int option, int value);
int dabnn_get_option(int option);

/* ceil(C / 64): 64-bit words per pixel for C channels.  Returns -1 if C <= 0. */
int64_t dabnn_packed_words(int64_t C);

/* Output extent of a convolution: floor((in + 2*pad - k) / stride) + 1, or -1 if the arguments
 * are invalid (in, k, stride <= 0, pad < 0, pad >= k, or in + 2*pad < k). */
int dabnn_conv_out_dim(int in, int k, int stride, int pad);

/*
 * Sign + bit-packing of an activation tensor (Sec. 2.1.1).
 *   x   : fp32  [n_pixels][C]              (NHWC with N*H*W flattened into n_pixels), read only
 *   out : u64   [n_pixels][ceil(C/64)]     written completely, tail bits 0
 * n_pixels may be 0: nothing is launched and the pointers are not looked at.
 * n_pixels * C must be < 2^40.
 */
int dabnn_bitpack(const float *x, uint64_t *out, int64_t n_pixels, int C, int sign_mode,
                  void *stream);

/*
 * Sign + bit-pack of an int32 tensor (Sec. 2.1.1: the sign bit of int32 and of IEEE-754 floats is
 * used alike): bit = 1 iff x < 0.  Same layout, arguments and errors as dabnn_bitpack; useful to
 * binarize an integer feature map (the output of dabnn_bconv2d) without a float detour.
 *   x : i32 [n_pixels][C] device        out : u64 [n_pixels][ceil(C/64)] device
 */
int dabnn_bitpack_i32(const int32_t *x, uint64_t *out, int64_t n_pixels, int C, void *stream);

/*
 * Layout conversion between this library's packed NHWC tensors and the paper's NC1HWC2 layout
 * (Sec. 2.1.2) with C2 = 128 bits, the format daBNN itself stores activations in:
 *   NHWC    : u64 [N][H][W][Cw]
 *   NC1HWC2 : u64 [N][C1][H][W][2],  C1 = ceil(Cw/2); for odd Cw the last group's second word is 0
 * Both device, both below 2^31 words; in and out must not overlap.
 */
int dabnn_nhwc_to_nc1hwc2(const uint64_t *in, uint64_t *out, int N, int H, int W, int Cw, void *stream);
int dabnn_nc1hwc2_to_nhwc(const uint64_t *in, uint64_t *out, int N, int H, int W, int Cw, void *stream);

/*
 * Fused batch-norm + shortcut + sign + bit-pack: the layer that sits between two binary
 * convolutions.  Sec. 2.1.1 (last sentence) names the fused BN-binarization layer; the blocks of
 * Bi-Real Net 18, the network of Sec. 2.3, add a real-valued shortcut before the next sign.  In
 * IEEE single precision, every operation rounded separately (no fused multiply-add):
 *
 *   z[p,c] = ((scale[c] * (float)y[p,c]) + shift[c]) + r[p,c]          (r term absent if r is NULL)
 *   bit    = IEEE sign bit of z            (the DABNN_SIGN_BIT rule; z = -0.0 packs as -1)
 *
 *   y     : i32 [n_pixels][C]  device   the output of dabnn_bconv2d
 *   scale, shift : f32 [C]     device   folded batch-norm (gamma/sqrt(var+eps), beta - mean*scale)
 *   r     : f32 [n_pixels][C]  device or NULL   the shortcut
 *   x_out : f32 [n_pixels][C]  device or NULL   receives z (the next block's shortcut); may equal r
 *   bits  : u64 [n_pixels][ceil(C/64)]  device, tail bits 0
 * One HBM-bound pass: 4 (+4 +4) + 1/8 bytes per element instead of a float pass plus a bit-pack.
 */
int dabnn_bn_sign_pack(const int32_t *y, const float *scale, const float *shift, const float *r,
                       float *x_out, uint64_t *bits, int64_t n_pixels, int C, void *stream);

/*
 * dabnn_bconv2d followed by dabnn_bn_sign_pack in one call, without the int32 feature map: a whole
 * Bi-Real-style block step (Sec. 2.3's network; Sec. 2.1.1's fused BN-binarization), bits in ->
 * next bits and next shortcut out.  Results are exactly those of the two calls in sequence.
 *   a, w         : as for dabnn_bconv2d
 *   scale, shift : f32 [Cout]            device
 *   r            : f32 [N][Ho][Wo][Cout] device or NULL (no shortcut)
 *   x_out        : f32 [N][Ho][Wo][Cout] device, required (it doubles as the staging buffer of the
 *                  int32 result for shapes the fused kernel does not cover); must not alias r
 *                  (dabnn_bn_sign_pack allows x_out == r; this call does not)
 *   bits         : u64 [N][Ho][Wo][ceil(Cout/64)] device, tail bits 0
 * The fused kernel runs 3x3 kernels, stride 1 or 2, up to 8 words per pixel (Cin <= 512), Cout % 64 == 0,
 * a shortcut, and scale, shift, r, x_out 16-byte aligned; every other valid case, and a launch with
 * fewer than about two 16-channel groups of work per SIMD (a single image, a small batch), runs as
 * the two kernels in sequence.
 */
int dabnn_bconv2d_bn_residual(const uint64_t *a, const uint64_t *w, const float *scale,
                              const float *shift, const float *r, float *x_out, uint64_t *bits,
                              int N, int H, int W, int Cin, int Cout, int kh, int kw, int stride,
                              int pad, void *stream);

/*
 * Ahead-of-time packing of binary-convolution weights (Sec. 3), same bit rule as above.
 *   w   : fp32 [Cout][kh][kw][Cin], any values (only the sign is used), read only
 *   out : u64  [Cout][kh][kw][ceil(Cin/64)]   -- the canonical packed weight layout
 */
int dabnn_pack_weights(const float *w, uint64_t *out, int Cout, int kh, int kw, int Cin,
                       int sign_mode, void *stream);

/*
 * Binary direct convolution (Sec. 2.1.2, Eq. 6-7; cross-correlation, no kernel flip).
 *   a : u64 [N][H][W][Cw]        packed activations, Cw = ceil(Cin/64), tail bits 0
 *   w : u64 [Cout][kh][kw][Cw]   packed weights (canonical layout), tail bits 0
 *   y : i32 [N][Ho][Wo][Cout]    Ho = dabnn_conv_out_dim(H, kh, stride, pad), same for Wo
 *
 *   y[n,ho,wo,co] = K - 2 * sum_{i,j,q} popcount(a[n, ho*stride-pad+i, wo*stride-pad+j, q]
 *                                              XOR w[co,i,j,q]),      K = kh*kw*Cin,
 * i.e. 2C - K with C the match count of Eq. 1.  A tap outside the image counts as an all-zero
 * word (every channel +1).  Tail bits must be 0 in both operands (true for buffers produced by
 * dabnn_bitpack / dabnn_pack_weights); they then cancel and K counts real channels only.
 * Requires 0 <= pad < min(kh, kw), stride >= 1, and every tensor below 2^31 elements.
 */
int dabnn_bconv2d(const uint64_t *a, const uint64_t *w, int32_t *y, int N, int H, int W, int Cin,
                  int Cout, int kh, int kw, int stride, int pad, void *stream);

/* Same operation with the kernel family chosen by the caller (a dabnn_algo).  Returns
 * DABNN_ERR_UNSUPPORTED, launching nothing, if that family cannot run the shape. */
int dabnn_bconv2d_algo(const uint64_t *a, const uint64_t *w, int32_t *y, int N, int H, int W,
                       int Cin, int Cout, int kh, int kw, int stride, int pad, int algo,
                       void *stream);

/*
 * BGEMM (Sec. 2.1.2, Eq. 1) on bit-packed matrices:
 *
 *   DABNN_BGEMM_MATCHES:  C[i][j] = sum_q bitcount(xnor(A[i][q], B[j][q])) restricted to the K real bits
 *                                 = K - sum_q popcount(A[i][q] XOR B[j][q])
 *   DABNN_BGEMM_SIGNED :  C[i][j] = K - 2 * sum_q popcount(A[i][q] XOR B[j][q])
 *
 *   A : u64 [M][Kw]  device, row-major; row i is the paper's A_{i,.}
 *   B : u64 [N][Kw]  device, row-major; row j is the paper's column B_{.,j}
 *   C : i32 [M][N]   device, written completely
 * Of the 64*Kw bits of a row the first K (0 < K <= 64*Kw, K < 2^23) are real; every other bit must
 * be 0 in both operands.  Kw need not be ceil(K/64): a patch-matrix row has kh*kw*ceil(Cin/64)
 * words holding kh*kw*Cin real bits.  Any shape runs; the fast kernel needs N % 16 == 0, C
 * 16-byte aligned and 2*Kw in {2,4,6,8,12,16,18,24,32,36,48,64,72,96,128,144}.
 */
int dabnn_bgemm(const uint64_t *A, const uint64_t *B, int32_t *C, int64_t M, int N, int Kw, int K,
                int mode, void *stream);

/*
 * Patch matrix (im2col) of a packed NHWC tensor: row (n,ho,wo) holds the kh*kw taps under that
 * output in (i, j) order, ceil(Cin/64) words each; a tap outside the image is an all-zero word
 * (+1 in every channel).  dabnn_bgemm of it with the packed filters [Cout][kh*kw*ceil(Cin/64)],
 * K = kh*kw*Cin, equals dabnn_bconv2d -- the BGEMM route that the paper measures its direct
 * convolution against (Fig. 4).
 *   a    : u64 [N][H][W][ceil(Cin/64)]                 device
 *   cols : u64 [N*Ho*Wo][kh*kw*ceil(Cin/64)]           device, written completely (< 2^31 words)
 */
int dabnn_im2col(const uint64_t *a, uint64_t *cols, int N, int H, int W, int Cin, int kh, int kw,
                 int stride, int pad, void *stream);

/*
 * Expanded-operand comparison route (not the default path).  CDNA4 has no 1-bit matrix
 * instruction, but +-1 is exact in int8: with every bit expanded to a byte the binary convolution
 * of Sec. 2.1.2 becomes an int8 implicit GEMM on the matrix cores, y = sum a*w with int32
 * accumulation, bit-identical to K - 2*popcount(a XOR w) of Eq. 6-7.  Provided so that the
 * XOR/popcount kernels can be measured against it, the 8x operand expansion included.
 *
 * dabnn_expand_int8: packed rows -> int8, +1 for bit 0 and -1 for bit 1.
 *   bits : u64 [rows][C/64]  device          out : i8 [rows][C]  device, 16-byte aligned
 *   C % 64 == 0 (DABNN_ERR_UNSUPPORTED otherwise).  Works for activations (rows = N*H*W) and for
 *   packed filters (rows = Cout*kh*kw) alike.
 * dabnn_bconv2d_int8: the convolution of dabnn_bconv2d on expanded operands.
 *   a8 : i8 [N][H][W][Cin]   w8 : i8 [Cout][kh][kw][Cin]   values +-1, device, 16-byte aligned
 *   y  : i32 [N][Ho][Wo][Cout]  device.  Out-of-image taps count as +1.
 *   Cin % 64 == 0 and Cout % 64 == 0 (DABNN_ERR_UNSUPPORTED otherwise); any kernel size, stride, pad.
 */
int dabnn_expand_int8(const uint64_t *bits, int8_t *out, int64_t rows, int C, void *stream);
int dabnn_bconv2d_int8(const int8_t *a8, const int8_t *w8, int32_t *y, int N, int H, int W, int Cin,
                       int Cout, int kh, int kw, int stride, int pad, void *stream);

/*
* Matrix-core route fed from the packed bits.  The same integers as dabnn_bconv2d (Sec. 2.1.2,
 * Eq. 6-7), computed as a matrix product: with a = 1 for an activation of -1 (else 0) and
 * s = +-1 for the weights, y = sum_k (1 - 2 a_k) s_k = S - 2 * sum_k a_k s_k, S = sum_k s_k.  The
 * activation operand is expanded from the packed words inside the kernel (one AND per operand
 * register), so the activations stay packed in memory; only the filters are expanded, once per
 * model, into the order in which the kernel consumes them.  `format` chooses the matrix
 * instruction: DABNN_MFMA_INT8 (v_mfma_i32_32x32x32_i8, one byte per weight) or DABNN_MFMA_FP4
 * (v_mfma_scale_f32_32x32x64_f8f6f4 on 4-bit E2M1 operands, one nibble per weight, fp32
 * accumulation of exact integers); a prepared buffer is used with the format it was made for.
 *
 * dabnn_mfma_weights_bytes: size in bytes of the prepared filter buffer for a layer, 0 if the
 *   shape or the format is outside what this route supports.
 * dabnn_prepare_weights_mfma:
 *   w  : u64 [Cout][3][3][Cin/64]  device, as written by dabnn_pack_weights
 *   wq : dabnn_mfma_weights_bytes(...) bytes, device, 16-byte aligned, written completely
 *        (operands in kernel order, then S[Cout] as int32); owned by the caller.
 * dabnn_bconv2d_mfma:
 *   a  : u64 [N][H][W][Cin/64]     device, as written by dabnn_bitpack
 *   wq : the prepared filters of the same layer shape and format
 *   y  : i32 [N][Ho][Wo][Cout]     device, written completely.  Out-of-image taps count as +1.
 * Supported: 3x3 kernels, stride 1 or 2, Cin in {64, 128, 256, 512}, Cout % 64 == 0 and at most
 * 8192, packed activations below 2^31 dwords; DABNN_ERR_UNSUPPORTED otherwise (nothing launched).
 */
typedef enum { DABNN_MFMA_INT8 = 0, DABNN_MFMA_FP4 = 1 } dabnn_mfma_format;
size_t dabnn_mfma_weights_bytes(int Cin, int Cout, int kh, int kw, int format);
int dabnn_prepare_weights_mfma(const uint64_t *w, void *wq, int Cin, int Cout, int kh, int kw,
                               int format, void *stream);
int dabnn_bconv2d_mfma(const uint64_t *a, const void *wq, int32_t *y, int N, int H, int W, int Cin,
                       int Cout, int kh, int kw, int stride, int pad, int format, void *stream);
/*
 * dabnn_bconv2d_bnsign (fused convolution + threshold + bit-pack, Sec. 2.1.1) on the matrix-core
 * route: same arguments and results, with the prepared filters `wq` in place of the packed ones,
 * and the shapes dabnn_bconv2d_mfma supports.  thr, flip: as written by dabnn_bn_thresholds.
 *   out : u64 [N][Ho][Wo][Cout/64]  device, written completely.
 */
int dabnn_bconv2d_bnsign_mfma(const uint64_t *a, const void *wq, const int32_t *thr,
                              const uint64_t *flip, uint64_t *out, int N, int H, int W, int Cin,
                              int Cout, int kh, int kw, int stride, int pad, int format, void *stream);

/*
 * Binary convolution with ZERO padding.  The paper builds its binary convolution on the standard
 * ONNX Sign and Convolution operators (Table 1 caption, Sec. 3), and ONNX Convolution pads with 0:
 * a tap outside the image contributes nothing, where dabnn_bconv2d counts it as +1 in every
 * channel.  Same arguments, layouts and constraints as dabnn_bconv2d;
 *
 *   y0[n,ho,wo,co] = sum over taps INSIDE the image of (Cin - 2 * popcount(a XOR w)),
 *
 * which equals dabnn_bconv2d's y minus (Cin - 2*popcount(w[co,i,j,:])) for every outside tap.
 * Interior outputs are identical; border outputs need not share K's parity.  Enqueues the
 * convolution and, for pad > 0, one in-place pass over the border outputs on the same stream.
 */
int dabnn_bconv2d_zeropad(const uint64_t *a, const uint64_t *w, int32_t *y, int N, int H, int W,
                          int Cin, int Cout, int kh, int kw, int stride, int pad, void *stream);

/*
 * Binary convolution fused with batch-norm and binarization: the output is the NEXT layer's packed
 * activation tensor, so neither the int32 feature map nor a separate bit-pack pass exists.  The
 * paper notes that its packing is compatible with a fused BN-binarization layer (Sec. 2.1.1, last
 * sentence); the layer computed here is sign(BN(conv)), expressed on the integer conv output y:
 *
 *   bit(n,ho,wo,co) = (y[n,ho,wo,co] < thr[co]) XOR flip bit co          (bit 1 <-> -1)
 *
 *   a, w  : as for dabnn_bconv2d
 *   thr   : i32 [Cout]            device, every value within [-2^30, 2^30]
 *   flip  : u64 [ceil(Cout/64)]   device, bit co%64 of word co/64, tail bits 0
 *   out   : u64 [N][Ho][Wo][ceil(Cout/64)]  device, written completely, tail bits 0
 * dabnn_bn_thresholds derives thr and flip from batch-norm parameters.
 */
int dabnn_bconv2d_bnsign(const uint64_t *a, const uint64_t *w, const int32_t *thr,
                         const uint64_t *flip, uint64_t *out, int N, int H, int W, int Cin,
                         int Cout, int kh, int kw, int stride, int pad, void *stream);

/*
 * HOST helper (every pointer is a HOST pointer; nothing is launched): integer thresholds that
 * reproduce, for every integer y in [-K, K], the sign of the inference-time batch-norm evaluated
 * in fp64,   z = gamma[c] * (y - mean[c]) / sqrt(var[c] + eps) + beta[c],   bit = 1 iff z < 0:
 *   (y < thr[c]) XOR flip bit c  ==  (z < 0).
 * gamma > 0 gives flip 0, gamma < 0 flip 1; gamma == 0 (or a NaN anywhere) gives a constant bit.
 *   gamma, beta, mean, var : f32 [Cout];  thr : i32 [Cout];  flip : u64 [ceil(Cout/64)]
 * Returns DABNN_ERR_NULL / DABNN_ERR_SHAPE (Cout <= 0, K <= 0 or K >= 2^30) like the other calls.
 */
int dabnn_bn_thresholds(const float *gamma, const float *beta, const float *mean, const float *var,
                        float eps, int Cout, int K, int32_t *thr, uint64_t *flip);

/* Which dabnn_algo DABNN_ALGO_AUTO resolves to for this shape with a 16-byte aligned y (no
 * launch); -1 if the shape is invalid. */
int dabnn_bconv2d_pick_algo(int N, int H, int W, int Cin, int Cout, int kh, int kw, int stride,
                            int pad);

/* Human-readable name of a dabnn_status; static storage, never NULL. */
const char *dabnn_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* DABNN_H */

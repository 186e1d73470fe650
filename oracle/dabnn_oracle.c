/*
 * CPU oracle for the daBNN hot path (arXiv 1908.05858): sign binarization, bit-packing and
 * binary convolution.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a slow, plain, obviously-correct
 * statement of what the GPU library must compute.  Only tests/, __graft_entry__.smoke() and the
 * cpu_baseline leg of bench.py may load it.  It shares no code, header, table or helper with the
 * HIP path and is never a fallback for it.
 *
 * The method reaches exactly (no approximation) a result with a plain definition, so every
 * function below is that definition written out:
 *
 *   - Sec. 2.1.1 (bit-packing): the binary value of an element is its existing IEEE-754 sign
 *     bit; N elements become an N-bit vector.
 *   - Sec. 2.1.2, Eq. 1 / Eq. 6-7: a binary convolution is sum_k bitcount(xnor(A, B)) with A the
 *     weights and B the im2col-ed input, which the paper says is the definition of convolution
 *     itself.  With K true bits per filter and C matching bits, the +-1 dot product is
 *     2C - K.  The oracle does not touch bits at all for the convolution: it multiplies and
 *     adds +-1.0f values, which is the textbook cross-correlation the bit formula must equal.
 *
 * Exactness of the float accumulation: every partial sum is an integer of magnitude
 * <= K = kh*kw*Cin.  The oracle refuses K >= 2^24, so fp32 represents every partial sum
 * exactly and any summation order gives the same value.
 *
 * Readings taken where the paper is silent (all restated in the project's design notes):
 *   - sign rule 0 (default, Sec. 2.1.1): -1 iff the sign bit is set (so -0.0 -> -1, NaN by its
 *     sign bit); sign rule 1: +1 iff x >= 0 (so -0.0 -> +1, NaN -> -1).
 *   - bit polarity: bit 1 <-> -1, bit 0 <-> +1.
 *   - bit order: channel c sits in 64-bit word c/64 at bit c%64 (LSB first); bits past the last
 *     channel are 0.
 *   - taps that fall outside the image have the value +1.
 *   - no kernel flip (cross-correlation); output size floor((in + 2*pad - k)/stride) + 1.
 *   - tensors: activations NHWC, weights [Cout][kh][kw][Cin].
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

#define ORACLE_OK 0
#define ORACLE_BAD_ARG 1

static float sign_value(float x, int sign_rule)
{
    if (sign_rule == 0)
        return signbit(x) ? -1.0f : 1.0f;
    return (x >= 0.0f) ? 1.0f : -1.0f;
}

/* s[i] = +1.0f or -1.0f, the binary value of x[i] (Sec. 2.1.1). */
int oracle_sign(const float *x, float *s, int64_t n, int sign_rule)
{
    if (!x || !s || n < 0 || (sign_rule != 0 && sign_rule != 1))
        return ORACLE_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        s[i] = sign_value(x[i], sign_rule);
    return ORACLE_OK;
}

/*
 * Bit-packing (Sec. 2.1.1): x is [n_pixels][C] fp32; out is [n_pixels][ceil(C/64)] words.
 * Bit (c % 64) of word (c / 64) is 1 iff the binary value of channel c is -1.
 */
int oracle_bitpack(const float *x, uint64_t *out, int64_t n_pixels, int C, int sign_rule)
{
    if (!x || !out || n_pixels < 0 || C <= 0 || (sign_rule != 0 && sign_rule != 1))
        return ORACLE_BAD_ARG;
    const int64_t words = ((int64_t)C + 63) / 64;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < n_pixels; ++p) {
        for (int64_t j = 0; j < words; ++j)
            out[p * words + j] = 0;
        for (int c = 0; c < C; ++c) {
            if (sign_value(x[p * (int64_t)C + c], sign_rule) < 0.0f)
                out[p * words + c / 64] |= (uint64_t)1 << (c % 64);
        }
    }
    return ORACLE_OK;
}

static int out_dim(int in, int k, int stride, int pad)
{
    if (in <= 0 || k <= 0 || stride <= 0 || pad < 0 || in + 2 * pad < k)
        return -1;
    return (in + 2 * pad - k) / stride + 1;
}

int oracle_conv_out_dim(int in, int k, int stride, int pad)
{
    return out_dim(in, k, stride, pad);
}

/* One output of the +-1 convolution (Eq. 6-7 read as the definition of convolution). */
static int32_t conv_one(const float *A, const float *Wt, int n, int ho, int wo, int co,
                        int H, int W, int Cin, int kh, int kw, int stride, int pad)
{
    float acc = 0.0f;
    for (int i = 0; i < kh; ++i) {
        const int hi = ho * stride - pad + i;
        for (int j = 0; j < kw; ++j) {
            const int wi = wo * stride - pad + j;
            const float *wrow = Wt + (((int64_t)co * kh + i) * kw + j) * Cin;
            if (hi >= 0 && hi < H && wi >= 0 && wi < W) {
                const float *arow = A + (((int64_t)n * H + hi) * W + wi) * Cin;
#pragma omp simd reduction(+ : acc)
                for (int c = 0; c < Cin; ++c)
                    acc += arow[c] * wrow[c];
            } else {
                /* outside the image every activation is +1 */
#pragma omp simd reduction(+ : acc)
                for (int c = 0; c < Cin; ++c)
                    acc += 1.0f * wrow[c];
            }
        }
    }
    return (int32_t)acc;
}

/*
 * Binary convolution on already-binarized tensors.
 *   A  : [N][H][W][Cin]      values +-1.0f
 *   Wt : [Cout][kh][kw][Cin] values +-1.0f
 *   Y  : [N][Ho][Wo][Cout]   int32
 */
int oracle_bconv2d(const float *A, const float *Wt, int32_t *Y, int N, int H, int W, int Cin,
                   int Cout, int kh, int kw, int stride, int pad)
{
    if (!A || !Wt || !Y || N <= 0 || Cin <= 0 || Cout <= 0)
        return ORACLE_BAD_ARG;
    const int Ho = out_dim(H, kh, stride, pad);
    const int Wo = out_dim(W, kw, stride, pad);
    if (Ho <= 0 || Wo <= 0 || (int64_t)kh * kw * Cin >= ((int64_t)1 << 24))
        return ORACLE_BAD_ARG;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int ho = 0; ho < Ho; ++ho) {
            for (int wo = 0; wo < Wo; ++wo) {
                int32_t *yrow = Y + (((int64_t)n * Ho + ho) * Wo + wo) * Cout;
                for (int co = 0; co < Cout; ++co)
                    yrow[co] = conv_one(A, Wt, n, ho, wo, co, H, W, Cin, kh, kw, stride, pad);
            }
        }
    }
    return ORACLE_OK;
}

/*
 * The same convolution evaluated only at n_samples chosen outputs:
 * idx is [n_samples][4] = (n, ho, wo, co); out[s] receives that output.
 */
int oracle_bconv2d_at(const float *A, const float *Wt, const int32_t *idx, int64_t n_samples,
                      int32_t *out, int N, int H, int W, int Cin, int Cout, int kh, int kw,
                      int stride, int pad)
{
    if (!A || !Wt || !idx || !out || n_samples < 0 || N <= 0 || Cin <= 0 || Cout <= 0)
        return ORACLE_BAD_ARG;
    const int Ho = out_dim(H, kh, stride, pad);
    const int Wo = out_dim(W, kw, stride, pad);
    if (Ho <= 0 || Wo <= 0 || (int64_t)kh * kw * Cin >= ((int64_t)1 << 24))
        return ORACLE_BAD_ARG;
    for (int64_t s = 0; s < n_samples; ++s) {
        const int32_t *q = idx + 4 * s;
        if (q[0] < 0 || q[0] >= N || q[1] < 0 || q[1] >= Ho || q[2] < 0 || q[2] >= Wo ||
            q[3] < 0 || q[3] >= Cout)
            return ORACLE_BAD_ARG;
    }
#pragma omp parallel for schedule(static)
    for (int64_t s = 0; s < n_samples; ++s) {
        const int32_t *q = idx + 4 * s;
        out[s] = conv_one(A, Wt, q[0], q[1], q[2], q[3], H, W, Cin, kh, kw, stride, pad);
    }
    return ORACLE_OK;
}

/*
 * The same convolution with ZERO padding, as the standard ONNX Convolution operator defines it
 * (the paper builds its binary convolution on the ONNX Sign and Convolution operators: Table 1
 * caption and Sec. 3): a tap outside the image contributes nothing, so border outputs are sums
 * over fewer than K products and need not share K's parity.  Inside the image A is +-1.0f.
 */
int oracle_bconv2d_zeropad(const float *A, const float *Wt, int32_t *Y, int N, int H, int W,
                           int Cin, int Cout, int kh, int kw, int stride, int pad)
{
    if (!A || !Wt || !Y || N <= 0 || Cin <= 0 || Cout <= 0)
        return ORACLE_BAD_ARG;
    const int Ho = out_dim(H, kh, stride, pad);
    const int Wo = out_dim(W, kw, stride, pad);
    if (Ho <= 0 || Wo <= 0 || (int64_t)kh * kw * Cin >= ((int64_t)1 << 24))
        return ORACLE_BAD_ARG;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int ho = 0; ho < Ho; ++ho) {
            for (int wo = 0; wo < Wo; ++wo) {
                for (int co = 0; co < Cout; ++co) {
                    float acc = 0.0f;
                    for (int i = 0; i < kh; ++i) {
                        const int hi = ho * stride - pad + i;
                        if (hi < 0 || hi >= H)
                            continue;
                        for (int j = 0; j < kw; ++j) {
                            const int wi = wo * stride - pad + j;
                            if (wi < 0 || wi >= W)
                                continue;
                            const float *arow = A + (((int64_t)n * H + hi) * W + wi) * Cin;
                            const float *wrow = Wt + (((int64_t)co * kh + i) * kw + j) * Cin;
                            for (int c = 0; c < Cin; ++c)
                                acc += arow[c] * wrow[c];
                        }
                    }
                    Y[(((int64_t)n * Ho + ho) * Wo + wo) * Cout + co] = (int32_t)acc;
                }
            }
        }
    }
    return ORACLE_OK;
}

/*
 * Bit-packing of int32 tensors (Sec. 2.1.1 uses the sign bit "in int32 and IEEE 754 float"
 * alike): bit = 1 iff x < 0, same word layout as oracle_bitpack.
 */
int oracle_bitpack_i32(const int32_t *x, uint64_t *out, int64_t n_pixels, int C)
{
    if (!x || !out || n_pixels < 0 || C <= 0)
        return ORACLE_BAD_ARG;
    const int words = (C + 63) / 64;
    for (int64_t p = 0; p < n_pixels; ++p) {
        for (int q = 0; q < words; ++q) {
            uint64_t wd = 0;
            for (int b = 0; b < 64; ++b) {
                const int c = 64 * q + b;
                if (c < C && x[p * C + c] < 0)
                    wd |= (uint64_t)1 << b;
            }
            out[p * words + q] = wd;
        }
    }
    return ORACLE_OK;
}

/*
 * NC1HWC2 layout of Sec. 2.1.2 with C2 = 128 bits (two 64-bit words): the channel words of a
 * pixel are split into C1 = ceil(Cw/2) groups and the group index becomes the second-slowest
 * dimension.   in : [N][H][W][Cw]   out : [N][C1][H][W][2]; a missing second word is 0.
 */
int oracle_nhwc_to_nc1hwc2(const uint64_t *in, uint64_t *out, int N, int H, int W, int Cw)
{
    if (!in || !out || N <= 0 || H <= 0 || W <= 0 || Cw <= 0)
        return ORACLE_BAD_ARG;
    const int C1 = (Cw + 1) / 2;
    for (int n = 0; n < N; ++n)
        for (int c1 = 0; c1 < C1; ++c1)
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    for (int k = 0; k < 2; ++k) {
                        const int q = 2 * c1 + k;
                        const uint64_t v =
                            q < Cw ? in[(((int64_t)n * H + h) * W + w) * Cw + q] : 0;
                        out[((((int64_t)n * C1 + c1) * H + h) * W + w) * 2 + k] = v;
                    }
    return ORACLE_OK;
}

/*
 * Fused batch-norm + binarization layer between two binary convolutions (Sec. 2.1.1, last
 * sentence, names the layer; Sec. 2.3 benchmarks Bi-Real Net 18, whose blocks add a real-valued
 * shortcut before the next sign).  Reading taken, in IEEE single precision with every operation
 * rounded separately (no fused multiply-add):
 *
 *   z[p,c] = ((scale[c] * (float)y[p,c]) + shift[c]) + r[p,c]        (r omitted when NULL)
 *   bit    = IEEE sign bit of z                                      (Sec. 2.1.1 sign rule)
 *
 * y is the integer convolution output, scale/shift the folded batch-norm.  z is written to
 * x_out when that is not NULL (the next block's shortcut); bits are packed like everywhere else.
 */
int oracle_bn_sign_pack(const int32_t *y, const float *scale, const float *shift, const float *r,
                        float *x_out, uint64_t *bits, int64_t n_pixels, int C)
{
    if (!y || !scale || !shift || !bits || n_pixels < 0 || C <= 0)
        return ORACLE_BAD_ARG;
    const int words = (C + 63) / 64;
    for (int64_t p = 0; p < n_pixels; ++p) {
        for (int q = 0; q < words; ++q)
            bits[p * words + q] = 0;
        for (int c = 0; c < C; ++c) {
            volatile float t = scale[c] * (float)y[p * C + c];  /* volatile: each step rounded */
            t = t + shift[c];
            if (r)
                t = t + r[p * C + c];
            const float z = t;
            if (x_out)
                x_out[p * C + c] = z;
            if (signbit(z))
                bits[p * words + c / 64] |= (uint64_t)1 << (c % 64);
        }
    }
    return ORACLE_OK;
}

/*
 * BGEMM (Sec. 2.1.2, Eq. 1) on already-binarized operands.
 *   A : [M][K] values +-1.0f          (row i is the paper's A_{i,.})
 *   B : [N][K] values +-1.0f          (row j is the paper's column B_{.,j})
 *   C : [M][N] int32
 * mode 1 is Eq. 1 as printed: C_ij = number of positions where the two vectors agree, i.e.
 * bitcount(xnor) over the K real bits.  mode 0 is the +-1 dot product that count stands for,
 * sum_k A_ik * B_jk = 2*C_ij - K, the quantity the convolution entry points return.
 */
int oracle_bgemm(const float *A, const float *B, int32_t *C, int64_t M, int N, int K, int mode)
{
    if (!A || !B || !C || M <= 0 || N <= 0 || K <= 0 || K >= (1 << 24) || (mode != 0 && mode != 1))
        return ORACLE_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        const float *a = A + i * K;
        for (int j = 0; j < N; ++j) {
            const float *b = B + (int64_t)j * K;
            if (mode == 1) {
                int32_t agree = 0;
                for (int k = 0; k < K; ++k)
                    agree += (a[k] == b[k]);
                C[i * N + j] = agree;
            } else {
                float acc = 0.0f;
                for (int k = 0; k < K; ++k)
                    acc += a[k] * b[k];
                C[i * N + j] = (int32_t)acc;
            }
        }
    }
    return ORACLE_OK;
}

/*
 * Binary convolution fused with batch-norm and binarization (Sec. 2.1.1, last sentence: the
 * packing scheme is compatible with a fused BN-binarization layer).  Reading taken: the layer is
 * sign(BN(conv)), with inference-time batch-norm per output channel evaluated in fp64,
 *
 *   z = gamma[co] * (y - mean[co]) / sqrt(var[co] + eps) + beta[co],     bit = 1 iff z < 0,
 *
 * where y is the integer convolution output above; z == 0 counts as +1 (bit 0).  The bits of a
 * pixel are packed like every other tensor here: channel co -> word co/64, bit co%64, tail 0.
 *   out : [N][Ho][Wo][ceil(Cout/64)] words
 */
int oracle_bconv2d_bnsign(const float *A, const float *Wt, const float *gamma, const float *beta,
                          const float *mean, const float *var, float eps, uint64_t *out, int N,
                          int H, int W, int Cin, int Cout, int kh, int kw, int stride, int pad)
{
    if (!A || !Wt || !gamma || !beta || !mean || !var || !out || N <= 0 || Cin <= 0 || Cout <= 0)
        return ORACLE_BAD_ARG;
    const int Ho = out_dim(H, kh, stride, pad);
    const int Wo = out_dim(W, kw, stride, pad);
    if (Ho <= 0 || Wo <= 0 || (int64_t)kh * kw * Cin >= ((int64_t)1 << 24))
        return ORACLE_BAD_ARG;
    const int words = (Cout + 63) / 64;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int ho = 0; ho < Ho; ++ho) {
            for (int wo = 0; wo < Wo; ++wo) {
                uint64_t *row = out + (((int64_t)n * Ho + ho) * Wo + wo) * words;
                for (int j = 0; j < words; ++j)
                    row[j] = 0;
                for (int co = 0; co < Cout; ++co) {
                    const int32_t yv =
                        conv_one(A, Wt, n, ho, wo, co, H, W, Cin, kh, kw, stride, pad);
                    const double z = (double)gamma[co] * ((double)yv - (double)mean[co]) /
                                         sqrt((double)var[co] + (double)eps) +
                                     (double)beta[co];
                    if (z < 0.0)
                        row[co / 64] |= (uint64_t)1 << (co % 64);
                }
            }
        }
    }
    return ORACLE_OK;
}

/*
 * Stand-in for the float glue between two binary convolutions of a Bi-Real-Net-18 body
 * (batch-norm plus shortcut), used only to GENERATE the next layer's fp32 input for the
 * full-network workload.  It is not part of the method under test; the GPU never computes it.
 *
 *   x_next[n,ho,wo,c] = gamma[c] * y[n,ho,wo,c] / sqrt(K) + beta[c] + shortcut[n,ho,wo,c]
 *
 * shortcut = x itself when stride == 1 (needs Cin == Cout, same spatial size), and for
 * stride == 2 the 2x2 average pool of x (window rows 2ho..2ho+1, cols 2wo..2wo+1, clipped to
 * the image) with its Cin channels repeated until Cout channels are filled (c -> c % Cin).
 * All arithmetic is fp32, evaluated in the order written.
 */
int oracle_glue(const float *x, const int32_t *y, const float *gamma, const float *beta,
                float *x_next, int N, int H, int W, int Cin, int Ho, int Wo, int Cout, int K,
                int stride)
{
    if (!x || !y || !gamma || !beta || !x_next || K <= 0)
        return ORACLE_BAD_ARG;
    if (stride == 1) {
        if (Cin != Cout || H != Ho || W != Wo)
            return ORACLE_BAD_ARG;
    } else if (stride == 2) {
        if (Ho != (H + 1) / 2 || Wo != (W + 1) / 2)
            return ORACLE_BAD_ARG;
    } else {
        return ORACLE_BAD_ARG;
    }
    const float inv = 1.0f / sqrtf((float)K);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int ho = 0; ho < Ho; ++ho) {
            for (int wo = 0; wo < Wo; ++wo) {
                const int64_t o = (((int64_t)n * Ho + ho) * Wo + wo) * Cout;
                for (int c = 0; c < Cout; ++c) {
                    float sc;
                    if (stride == 1) {
                        sc = x[(((int64_t)n * H + ho) * W + wo) * Cin + c];
                    } else {
                        float sum = 0.0f;
                        int cnt = 0;
                        for (int di = 0; di < 2; ++di) {
                            for (int dj = 0; dj < 2; ++dj) {
                                const int hi = 2 * ho + di, wi = 2 * wo + dj;
                                if (hi < H && wi < W) {
                                    sum += x[(((int64_t)n * H + hi) * W + wi) * Cin + c % Cin];
                                    ++cnt;
                                }
                            }
                        }
                        sc = sum / (float)cnt;
                    }
                    x_next[o + c] = gamma[c] * ((float)y[o + c] * inv) + beta[c] + sc;
                }
            }
        }
    }
    return ORACLE_OK;
}

// Zero-padding correction for the binary convolution.
//
// The convolution kernels treat a tap outside the image as an all-zero word, i.e. as +1 in every
// channel.  The ONNX Convolution operator, which the paper's binary convolution is built on
// (Table 1 caption, Sec. 3), pads with 0 instead: an outside tap contributes nothing.  The two
// differ, at border outputs only, by the plain sum of the weights under the outside taps,
//
//   y0[n,ho,wo,co] = y[n,ho,wo,co] - sum_{(i,j) outside} (Cin - 2*popcount(w[co,i,j,:])),
//
// which depends on the output's border class and on co but not on the image.  The kernel below
// applies that correction in place, touching border pixels only.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "launch.h"

namespace dabnn {
namespace {

// Outputs whose window leaves the image along one axis: a prefix [0, lo) and a suffix [hi, n_out).
struct BorderAxis {
    int lo, hi, count;  // count = lo + (n_out - hi)
};

BorderAxis border_axis(int in, int n_out, int k, int stride, int pad)
{
    // o*stride - pad < 0  <=>  o < ceil(pad/stride);   o*stride - pad + k - 1 >= in  <=>
    // o >= ceil((in - k + 1 + pad)/stride)
    int lo = (pad + stride - 1) / stride;
    if (lo > n_out)
        lo = n_out;
    const int first_bad = in - k + 1 + pad;  // may be <= 0 for an image narrower than the kernel
    int hi = first_bad <= 0 ? 0 : (first_bad + stride - 1) / stride;
    if (hi < lo)
        hi = lo;
    if (hi > n_out)
        hi = n_out;
    return BorderAxis{lo, hi, lo + (n_out - hi)};
}

// One thread per (border pixel of an image, output channel); it derives its correction once and
// applies it to that pixel of every image in [n_begin, n_end).  Consecutive threads are
// consecutive channels, so every read-modify-write of y is coalesced.
__global__ __launch_bounds__(256) void bconv_zeropad_fix_kernel(
    const uint64_t* __restrict__ w, int32_t* __restrict__ y, ConvShape s, BorderAxis rows,
    BorderAxis cols, int border_pixels, int images_per_block)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (e >= static_cast<int64_t>(border_pixels) * s.Cout)
        return;
    const int co = static_cast<int>(e % s.Cout);
    const int b = static_cast<int>(e / s.Cout);
    // border pixels of one image: first every pixel of the bad rows, then the bad columns of the
    // remaining rows
    int ho, wo;
    const int in_bad_rows = rows.count * s.Wo;
    if (b < in_bad_rows) {
        const int r = b / s.Wo;
        wo = b - r * s.Wo;
        ho = r < rows.lo ? r : rows.hi + (r - rows.lo);
    } else {
        const int q = b - in_bad_rows;
        const int r = q / cols.count;
        const int c = q - r * cols.count;
        ho = rows.lo + r;
        wo = c < cols.lo ? c : cols.hi + (c - cols.lo);
    }
    int corr = 0;
    for (int i = 0; i < s.kh; ++i) {
        const int hi = ho * s.stride - s.pad + i;
        for (int j = 0; j < s.kw; ++j) {
            const int wi = wo * s.stride - s.pad + j;
            if (hi >= 0 && hi < s.H && wi >= 0 && wi < s.W)
                continue;
            const uint64_t* wp = w + ((static_cast<int64_t>(co) * s.kh + i) * s.kw + j) * s.Cw;
            int minus = 0;  // tail bits are 0, so this counts -1 weights of real channels only
            for (int q = 0; q < s.Cw; ++q)
                minus += __popcll(wp[q]);
            corr += s.Cin - 2 * minus;
        }
    }
    const int n_begin = blockIdx.y * images_per_block;
    const int n_end = min(s.N, n_begin + images_per_block);
    const int64_t image_stride = static_cast<int64_t>(s.Ho) * s.Wo * s.Cout;
    int32_t* p = y + n_begin * image_stride + (static_cast<int64_t>(ho) * s.Wo + wo) * s.Cout + co;
    for (int n = n_begin; n < n_end; ++n, p += image_stride)
        *p -= corr;
}

}  // namespace

hipError_t launch_bconv_zeropad_fix(const uint64_t* w, int32_t* y, const ConvShape& s,
                                    hipStream_t stream)
{
    const BorderAxis rows = border_axis(s.H, s.Ho, s.kh, s.stride, s.pad);
    const BorderAxis cols = border_axis(s.W, s.Wo, s.kw, s.stride, s.pad);
    const int64_t border_pixels =
        static_cast<int64_t>(rows.count) * s.Wo + static_cast<int64_t>(s.Ho - rows.count) * cols.count;
    if (border_pixels == 0)
        return hipSuccess;  // no window leaves the image (pad == 0)
    const int64_t per_image = border_pixels * s.Cout;  // < 2^31: not more than one image's outputs
    const int64_t blocks_x = (per_image + 255) / 256;
    // enough blocks to fill the chip, each thread still amortising its correction over images
    int64_t chunks = (4096 + blocks_x - 1) / blocks_x;
    if (chunks > s.N)
        chunks = s.N;
    if (chunks > 65535)
        chunks = 65535;
    const int images_per_block = static_cast<int>((s.N + chunks - 1) / chunks);
    const unsigned grid_y = static_cast<unsigned>((s.N + images_per_block - 1) / images_per_block);
    bconv_zeropad_fix_kernel<<<dim3(static_cast<unsigned>(blocks_x), grid_y), dim3(256), 0, stream>>>(
        w, y, s, rows, cols, static_cast<int>(border_pixels), images_per_block);
    return hipGetLastError();
}

}  // namespace dabnn

// Expanded-operand comparison route for the binary convolution (Sec. 2.1.2, Eq. 6-7 give the
// result; this file computes the same integers another way).
//
// CDNA4 has no 1-bit matrix instruction, so the library's convolution is XOR + popcount on the
// vector ALU.  The matrix cores do take int8, and +-1 is exact in int8: expanding every bit to a
// byte (8x the operand bytes) turns the binary convolution into an ordinary int8 implicit GEMM
// with int32 accumulation, y = sum a*w, bit-identical to K - 2*popcount(a XOR w).  It is built to
// be measured against the XOR/popcount kernels with the expansion cost in view, not as the
// default path.
//
//   expand_pm1_kernel : packed bits -> int8 (+1 for bit 0, -1 for bit 1), activations and filters
//   bconv_mfma_i8_kernel : block tile (64*WM pixels) x (64*WN channels), four wavefronts, each a
//       64 x 64 tile = 2 x 2 v_mfma_i32_32x32x32_i8 accumulators.  The K dimension runs over
//       (tap, 64-channel slab); per step the block stages a [pixels][64 B] and a [channels][64 B]
//       tile in LDS (80-byte row pitch: conflict-free 16-byte reads) while the next step's global
//       loads are already in flight.  Out-of-image taps are staged as +1 bytes.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "launch.h"

namespace dabnn {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Four bits -> four bytes, 0x01 for a 0 bit and 0xFF for a 1 bit.  The multiply places bit j at
// bit 8j (the four shifted copies do not overlap, so nothing carries); x*255 turns each 0/1 byte
// into 0x00/0xFF without borrowing across bytes.
__device__ __forceinline__ uint32_t expand_nibble(uint32_t nib)
{
    const uint32_t spread = __umul24(nib, 0x204081u) & 0x01010101u;
    return ((spread << 8) - spread) | 0x01010101u;
}

// One thread per 16 channels of a row: 16 bits in, one 16-byte store out.  C % 64 == 0.
__global__ __launch_bounds__(256) void expand_pm1_kernel(const uint64_t* __restrict__ bits,
                                                         int8_t* __restrict__ out, int64_t total16)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (idx >= total16)
        return;
    // 16-channel group idx of the flattened tensor lives in word idx/4, bits 16*(idx%4)..+15
    const uint32_t b16 = static_cast<uint32_t>(bits[idx >> 2] >> (16 * (idx & 3))) & 0xffffu;
    v4i v;
    v.x = static_cast<int>(expand_nibble(b16 & 15u));
    v.y = static_cast<int>(expand_nibble((b16 >> 4) & 15u));
    v.z = static_cast<int>(expand_nibble((b16 >> 8) & 15u));
    v.w = static_cast<int>(expand_nibble(b16 >> 12));
    reinterpret_cast<v4i*>(out)[idx] = v;
}

constexpr int kPitch = 80;  // bytes per LDS row: 64 of data + 16 of padding

template <int WM, int WN>  // wavefronts along pixels and channels, WM * WN == 4
__global__ __launch_bounds__(256) void bconv_mfma_i8_kernel(const int8_t* __restrict__ a8,
                                                            const int8_t* __restrict__ w8,
                                                            int32_t* __restrict__ y, ConvShape s,
                                                            int total_pix)
{
    constexpr int BM = 64 * WM, BN = 64 * WN;
    constexpr int ACH = BM * 4 / 256;  // 16-byte chunks of the pixel tile per thread
    constexpr int BCH = BN * 4 / 256;  // 16-byte chunks of the channel tile per thread
    __shared__ __attribute__((aligned(16))) int8_t lds_a[BM * kPitch];
    __shared__ __attribute__((aligned(16))) int8_t lds_b[BN * kPitch];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = t >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int pix0 = blockIdx.x * BM;
    const int cout0 = blockIdx.y * BN;

    // The chunks this thread stages: chunk c = t + 256*r covers row c/4, bytes 16*(c%4)..+15.
    int a_hi0[ACH], a_wi0[ACH], a_img[ACH];
    for (int r = 0; r < ACH; ++r) {
        const int row = (t + 256 * r) >> 2;
        const int p = min(pix0 + row, total_pix - 1);  // rows past the end repeat the last pixel
        const int n = p / (s.Ho * s.Wo);
        const int rem = p - n * (s.Ho * s.Wo);
        const int ho = rem / s.Wo;
        a_hi0[r] = ho * s.stride - s.pad;
        a_wi0[r] = (rem - ho * s.Wo) * s.stride - s.pad;
        a_img[r] = n * s.H;
    }
    const int part = (t & 3) * 16;
    const int slabs = s.Cin / 64;
    const int steps = s.kh * s.kw * slabs;
    const int64_t w_row = static_cast<int64_t>(s.kh) * s.kw * s.Cin;  // bytes per filter

    v4i a_regs[ACH], b_regs[BCH];
    auto load_step = [&](int step) {
        const int tap = step / slabs;
        const int slab = step - tap * slabs;
        const int i = tap / s.kw, j = tap - i * s.kw;
        for (int r = 0; r < ACH; ++r) {
            const int hi = a_hi0[r] + i, wi = a_wi0[r] + j;
            if (hi >= 0 && hi < s.H && wi >= 0 && wi < s.W) {
                const int64_t off =
                    (static_cast<int64_t>(a_img[r] + hi) * s.W + wi) * s.Cin + slab * 64 + part;
                a_regs[r] = *reinterpret_cast<const v4i*>(a8 + off);
            } else {
                a_regs[r] = v4i{0x01010101, 0x01010101, 0x01010101, 0x01010101};  // +1 padding
            }
        }
        for (int r = 0; r < BCH; ++r) {
            const int row = (t + 256 * r) >> 2;
            const int64_t off = (cout0 + row) * w_row + static_cast<int64_t>(tap) * s.Cin + slab * 64 + part;
            b_regs[r] = *reinterpret_cast<const v4i*>(w8 + off);
        }
    };

    v16i acc[2][2] = {};
    load_step(0);
    for (int step = 0; step < steps; ++step) {
        __syncthreads();  // every wavefront is done reading the previous tiles
        for (int r = 0; r < ACH; ++r)
            *reinterpret_cast<v4i*>(lds_a + ((t + 256 * r) >> 2) * kPitch + part) = a_regs[r];
        for (int r = 0; r < BCH; ++r)
            *reinterpret_cast<v4i*>(lds_b + ((t + 256 * r) >> 2) * kPitch + part) = b_regs[r];
        __syncthreads();
        if (step + 1 < steps)
            load_step(step + 1);  // in flight while the matrix cores work
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            // lane l feeds row l%32 with bytes 16*(l/32)..+15 of this 32-wide K slice; the same
            // K assignment is used for both operands, which is all the dot product needs
            const int col = kk * 32 + (lane >> 5) * 16;
            v4i af[2], bf[2];
#pragma unroll
            for (int m = 0; m < 2; ++m)
                af[m] = *reinterpret_cast<const v4i*>(lds_a + (wm * 64 + m * 32 + (lane & 31)) * kPitch + col);
#pragma unroll
            for (int n = 0; n < 2; ++n)
                bf[n] = *reinterpret_cast<const v4i*>(lds_b + (wn * 64 + n * 32 + (lane & 31)) * kPitch + col);
#pragma unroll
            for (int m = 0; m < 2; ++m)
#pragma unroll
                for (int n = 0; n < 2; ++n)
                    acc[m][n] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[m], bf[n], acc[m][n], 0, 0, 0);
        }
    }

    // Accumulator register v of lane l is C[8*(v/4) + 4*(l/32) + v%4][l%32]: lanes 0..31 of one
    // store instruction write 32 consecutive channels (128 bytes) of one pixel.
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int n = 0; n < 2; ++n)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int p = pix0 + wm * 64 + m * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v & 3);
                const int co = cout0 + wn * 64 + n * 32 + (lane & 31);
                if (p < total_pix)
                    y[static_cast<int64_t>(p) * s.Cout + co] = acc[m][n][v];
            }
}

}  // namespace

hipError_t launch_expand_pm1(const uint64_t* bits, int8_t* out, int64_t rows, int C,
                             hipStream_t stream)
{
    if (C % 64 != 0)
        return hipErrorNotSupported;
    const int64_t total16 = rows * (C / 16);
    const int64_t blocks = (total16 + 255) / 256;
    if (blocks > 0x7fffffff)
        return hipErrorNotSupported;
    expand_pm1_kernel<<<dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream>>>(bits, out, total16);
    return hipGetLastError();
}

bool bconv_mfma_supports(const ConvShape& s)
{
    return s.Cin % 64 == 0 && s.Cout % 64 == 0;
}

hipError_t launch_bconv_mfma_i8(const int8_t* a8, const int8_t* w8, int32_t* y, const ConvShape& s,
                                hipStream_t stream)
{
    if (!bconv_mfma_supports(s))
        return hipErrorNotSupported;
    const int64_t total_pix = static_cast<int64_t>(s.N) * s.Ho * s.Wo;  // < 2^31 (checked by the caller)
    if (s.Cout % 128 == 0) {
        const dim3 grid(static_cast<unsigned>((total_pix + 127) / 128), static_cast<unsigned>(s.Cout / 128));
        bconv_mfma_i8_kernel<2, 2><<<grid, dim3(256), 0, stream>>>(a8, w8, y, s, static_cast<int>(total_pix));
    } else {
        const dim3 grid(static_cast<unsigned>((total_pix + 255) / 256), static_cast<unsigned>(s.Cout / 64));
        bconv_mfma_i8_kernel<4, 1><<<grid, dim3(256), 0, stream>>>(a8, w8, y, s, static_cast<int>(total_pix));
    }
    return hipGetLastError();
}

}  // namespace dabnn

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
//       (tap, 64-channel slab) pieces; per step the block stages a [pixels][64 or 128 B] and a
//       [channels][64 or 128 B] tile in LDS (row pitch + 16 bytes: conflict-free 16-byte reads)
//       while the next step's global loads are already in flight.  Out-of-image taps are staged
//       as +1 bytes.
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

// WM x WN wavefronts along pixels and channels (WM * WN == 4); PIECES 64-byte K pieces per step.
template <int WM, int WN, int PIECES>
__global__ __launch_bounds__(256) void bconv_mfma_i8_kernel(const int8_t* __restrict__ a8,
                                                            const int8_t* __restrict__ w8,
                                                            int32_t* __restrict__ y, ConvShape s,
                                                            int total_pix)
{
    constexpr int BM = 64 * WM, BN = 64 * WN;
    constexpr int kStepBytes = 64 * PIECES;  // K bytes staged per step
    constexpr int kPitch = kStepBytes + 16;  // bytes per LDS row; the 16-byte pad keeps 16-byte
                                             // reads of consecutive rows on distinct banks
    constexpr int CPR = 4 * PIECES;          // 16-byte chunks per staged row
    constexpr int RPP = 256 / CPR;           // rows staged per pass of the 256 threads
    constexpr int ACH = BM / RPP;            // chunks of the pixel tile per thread
    constexpr int BCH = BN / RPP;            // chunks of the channel tile per thread
    __shared__ __attribute__((aligned(16))) int8_t lds_a[BM * kPitch];
    __shared__ __attribute__((aligned(16))) int8_t lds_b[BN * kPitch];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = t >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int pix0 = blockIdx.x * BM;
    const int cout0 = blockIdx.y * BN;

    // The K dimension is a list of 64-byte pieces (tap, 64-channel slab), tap-major -- which is
    // also the byte order of a filter.  A step stages PIECES consecutive pieces.  Thread t stages,
    // for rows t/CPR + RPP*r, the 16 bytes at `part` of piece `half` of the step.
    const int half = (t >> 2) & (PIECES - 1);
    const int part = (t & 3) * 16;
    const int slabs = s.Cin / 64;
    const int n_pieces = s.kh * s.kw * slabs;
    const int steps = (n_pieces + PIECES - 1) / PIECES;

    // Per staged pixel row: byte offset of the window's top-left tap (may point outside the
    // tensor; only used for taps inside the image) and one validity bit per tap.
    int a_base[ACH];
    uint32_t a_valid[ACH];
#pragma unroll
    for (int r = 0; r < ACH; ++r) {
        const int p = min(pix0 + t / CPR + RPP * r, total_pix - 1);  // rows past the end repeat
        const int n = p / (s.Ho * s.Wo);
        const int rem = p - n * (s.Ho * s.Wo);
        const int ho = rem / s.Wo;
        const int hi0 = ho * s.stride - s.pad;
        const int wi0 = (rem - ho * s.Wo) * s.stride - s.pad;
        a_base[r] = ((n * s.H + hi0) * s.W + wi0) * s.Cin + part;
        uint32_t m = 0;
        for (int i = 0; i < s.kh; ++i)
            for (int j = 0; j < s.kw; ++j)
                if (hi0 + i >= 0 && hi0 + i < s.H && wi0 + j >= 0 && wi0 + j < s.W)
                    m |= 1u << (i * s.kw + j);
        a_valid[r] = m;
    }
    int b_base[BCH];
#pragma unroll
    for (int r = 0; r < BCH; ++r)
        b_base[r] = (cout0 + t / CPR + RPP * r) * (s.kh * s.kw * s.Cin) + part;

    // (tap row, tap column, slab) of this thread's piece of the current step
    int piece = half, ti = 0, tj = 0, slab = half;
    auto normalise = [&]() {
        while (slab >= slabs) {
            slab -= slabs;
            if (++tj == s.kw) {
                tj = 0;
                ++ti;
            }
        }
    };
    normalise();

    v4i a_regs[ACH], b_regs[BCH];
    auto load_step = [&]() {
        const bool live = piece < n_pieces;  // the last step may be only partly filled
        const int tap = ti * s.kw + tj;
        const int a_off = (ti * s.W + tj) * s.Cin + slab * 64;
#pragma unroll
        for (int r = 0; r < ACH; ++r) {
            if (!live)
                a_regs[r] = v4i{0, 0, 0, 0};  // contributes nothing
            else if ((a_valid[r] >> tap) & 1u)
                a_regs[r] = *reinterpret_cast<const v4i*>(a8 + (a_base[r] + a_off));
            else
                a_regs[r] = v4i{0x01010101, 0x01010101, 0x01010101, 0x01010101};  // +1 padding
        }
#pragma unroll
        for (int r = 0; r < BCH; ++r) {
            if (live)
                b_regs[r] = *reinterpret_cast<const v4i*>(w8 + (b_base[r] + piece * 64));
            else
                b_regs[r] = v4i{0, 0, 0, 0};
        }
        piece += PIECES;
        slab += PIECES;
        normalise();
    };

    const int stage_off = (t / CPR) * kPitch + half * 64 + part;
    v16i acc[2][2] = {};
    load_step();
    for (int step = 0; step < steps; ++step) {
        __syncthreads();  // every wavefront is done reading the previous tiles
#pragma unroll
        for (int r = 0; r < ACH; ++r)
            *reinterpret_cast<v4i*>(lds_a + stage_off + RPP * r * kPitch) = a_regs[r];
#pragma unroll
        for (int r = 0; r < BCH; ++r)
            *reinterpret_cast<v4i*>(lds_b + stage_off + RPP * r * kPitch) = b_regs[r];
        __syncthreads();
        if (step + 1 < steps)
            load_step();  // in flight while the matrix cores work
#pragma unroll
        for (int kk = 0; kk < kStepBytes / 32; ++kk) {
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
    // one validity bit per tap in a 32-bit mask; 32-bit byte offsets into both operands
    return s.Cin % 64 == 0 && s.Cout % 64 == 0 && s.kh * s.kw <= 32;
}

hipError_t launch_bconv_mfma_i8(const int8_t* a8, const int8_t* w8, int32_t* y, const ConvShape& s,
                                hipStream_t stream)
{
    if (!bconv_mfma_supports(s))
        return hipErrorNotSupported;
    const int64_t total_pix = static_cast<int64_t>(s.N) * s.Ho * s.Wo;  // < 2^31 (checked by the caller)
    if (s.Cout % 128 == 0) {
        const dim3 grid(static_cast<unsigned>((total_pix + 127) / 128), static_cast<unsigned>(s.Cout / 128));
        if (s.Cin >= 128)
            bconv_mfma_i8_kernel<2, 2, 2><<<grid, dim3(256), 0, stream>>>(a8, w8, y, s, static_cast<int>(total_pix));
        else
            bconv_mfma_i8_kernel<2, 2, 1><<<grid, dim3(256), 0, stream>>>(a8, w8, y, s, static_cast<int>(total_pix));
    } else {
        const dim3 grid(static_cast<unsigned>((total_pix + 255) / 256), static_cast<unsigned>(s.Cout / 64));
        if (s.Cin >= 128)
            bconv_mfma_i8_kernel<4, 1, 2><<<grid, dim3(256), 0, stream>>>(a8, w8, y, s, static_cast<int>(total_pix));
        else
            bconv_mfma_i8_kernel<4, 1, 1><<<grid, dim3(256), 0, stream>>>(a8, w8, y, s, static_cast<int>(total_pix));
    }
    return hipGetLastError();
}

}  // namespace dabnn

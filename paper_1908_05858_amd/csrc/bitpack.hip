// Sign + bit-packing of fp32 rows into 64-bit words (Sec. 2.1.1), for gfx950 wave64.
//
// The paper gathers sign bits with ARM's shift-right-insert so that many elements are packed
// per instruction and no element is compared with zero.  The wave64 equivalent used here: lane i
// of a wavefront loads channel 64*j + i of a pixel (one fully coalesced 256-byte read per
// wavefront), and ONE vector compare on the raw fp32 bits writes all 64 sign bits into a scalar
// register pair -- that pair already is the packed word, least significant bit = lowest channel.
// Eight such words are built per wavefront from eight independent loads in flight, moved into
// lanes 0..7 with a lane select, and stored as one contiguous 64-byte write (measured on MI355X:
// 8 words per wavefront 6.65 TB/s on an 848 MB pass, 16 words 6.4, 32 words 6.15, 4 words 5.9).
//
// The kernel is bound by HBM reads: 4 bytes read and 1/8 byte written per element.
#include "kernel_util.h"
#include "launch.h"

namespace dabnn {
namespace {

constexpr int kWordsPerWave = 8;
constexpr int kWavesPerBlock = 4;

// Bit value (1 <-> -1) from the raw fp32 bits, integer-only so that denormal flushing modes
// cannot change the result.
template <int MODE>
__device__ __forceinline__ bool negative_bit(uint32_t u)
{
    if (MODE == 0)
        return static_cast<int32_t>(u) < 0;  // the IEEE sign bit itself
    // !(x >= 0): any negative non-zero value (this includes NaNs with the sign set), or a NaN.
    return (u > 0x80000000u) || ((u & 0x7fffffffu) > 0x7f800000u);
}

// FLAT: C is a multiple of 64, so word g covers the 64 consecutive floats starting at 64*g.
template <int MODE, bool FLAT>
__global__ __launch_bounds__(64 * kWavesPerBlock) void bitpack_kernel(
    const uint32_t* __restrict__ x, uint2* __restrict__ out, int64_t n_words, int C, int Cw)
{
    const int lane = threadIdx.x & 63;
    const int wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t g0 =
        (static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave_in_block) * kWordsPerWave;
    if (g0 >= n_words)
        return;

    uint32_t v[kWordsPerWave];
    if (FLAT) {
        if (g0 + kWordsPerWave <= n_words) {
            const uint32_t* src = x + g0 * 64 + lane;
#pragma unroll
            for (int k = 0; k < kWordsPerWave; ++k)
                v[k] = __builtin_nontemporal_load(src + k * 64);
        } else {
#pragma unroll
            for (int k = 0; k < kWordsPerWave; ++k)
                v[k] = (g0 + k < n_words) ? x[(g0 + k) * 64 + lane] : 0u;
        }
    } else {
        int64_t p = g0 / Cw;
        int j = static_cast<int>(g0 - p * Cw);
#pragma unroll
        for (int k = 0; k < kWordsPerWave; ++k) {
            const int c = 64 * j + lane;
            const bool valid = (g0 + k < n_words) && (c < C);
            v[k] = valid ? x[p * C + c] : 0u;  // a missing channel packs as bit 0
            if (++j == Cw) {
                j = 0;
                ++p;
            }
        }
    }

    uint32_t lo = 0, hi = 0;
    static_for<0, kWordsPerWave>([&](auto kc) {
        constexpr int k = decltype(kc)::value;
        // the 64 sign bits of word k, wave-uniform; lane k keeps them for the store
        const uint64_t word = __builtin_amdgcn_ballot_w64(negative_bit<MODE>(v[k]));
        if (lane == k) {
            lo = static_cast<uint32_t>(word);
            hi = static_cast<uint32_t>(word >> 32);
        }
    });
    if (lane < kWordsPerWave && g0 + lane < n_words)
        out[g0 + lane] = make_uint2(lo, hi);
}

// C not a multiple of 64.  Rows are then not aligned to the 256-byte runs a wavefront reads best,
// and a pixel's last word has only C % 64 real channels.  Instead of reading row by row with
// masked lanes, the tensor is read as ONE flat stream of floats in aligned 64-element chunks
// (every load a full coalesced 256-byte run); each chunk's 64 sign bits form a ballot, and an
// output word is a bit-field of that flat bit stream: word (p, j) starts at flat bit p*C + 64*j
// and is min(64, C - 64*j) bits long.
//
// A wavefront owns 32 consecutive chunks (8 KB of input, whatever C is) and produces the words
// that START in them: it loads those chunks and the next one (a word may end there), parks ballot
// k in lane k (v_writelane), and lane l then assembles its word from two neighbouring ballots
// with a funnel shift and a length mask; 64 words per pass, as many passes as the chunks hold
// word starts (one for C >= 32).  The first word that starts at or after flat bit B is
// (B / C) * Cw + ceil((B % C) / 64).
//
// Every output word uses exactly the flat bits [start, start + len), all of them inside the
// tensor, so whatever the clamped loads at the tensor's end bring in is shifted or masked away.
//
// The kernel is built to issue few instructions, because at 33 loads per 8 KB the instruction
// count, not HBM, bounds it otherwise: everything per wavefront is scalar, the loads of a
// wavefront inside the tensor share one scalar base address and differ in their immediate
// offsets, and divisions are a multiply and a shift.  WIDE = false covers tensors below 2^31
// elements in 32-bit arithmetic; WIDE = true does the per-wavefront part in 64 bits (real
// divisions) for anything larger.
constexpr int kTailChunks = 32;

// Lane K of `blo` / `bhi` takes the scalars `lo` / `hi` (v_writelane_b32).  The scalars come from
// a vector compare just before; gfx950 wants wait states between a vector instruction's write of
// a scalar register and a vector instruction's read of it, which the compiler cannot see inside
// an asm statement, so the statement brings its own (4).
template <int K>
__device__ __forceinline__ void park_in_lane(int& blo, int& bhi, uint32_t lo, uint32_t hi)
{
    asm("s_nop 3\n\tv_writelane_b32 %0, %2, %4\n\tv_writelane_b32 %1, %3, %4"
        : "+v"(blo), "+v"(bhi)
        : "s"(lo), "s"(hi), "n"(K));
}

struct TailArgs {
    int64_t n_words, n_floats;
    int C, Cw;
    uint32_t c_mul, c_shift;    // fast_div constants of C
    uint32_t cw_mul, cw_shift;  // ... of Cw
};

template <int MODE, bool WIDE>
__global__ __launch_bounds__(64 * kWavesPerBlock) void bitpack_tail_kernel(
    const uint32_t* __restrict__ x, uint2* __restrict__ out, const TailArgs a)
{
    using index_t = std::conditional_t<WIDE, int64_t, uint32_t>;
    const index_t n_words = static_cast<index_t>(a.n_words);
    const index_t n_floats = static_cast<index_t>(a.n_floats);
    const int C = a.C, Cw = a.Cw;
    const int lane = threadIdx.x & 63;
    const int wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const index_t c0 =
        (static_cast<index_t>(blockIdx.x) * kWavesPerBlock + wave_in_block) * kTailChunks;
    const index_t B0 = c0 * 64;   // first flat bit (= element) of this wavefront
    if (B0 >= n_floats)
        return;

    // pixel of flat bit B, and the first word that starts at or after B
    auto pixel_of = [&](index_t B) -> index_t {
        if constexpr (WIDE)
            return B / C;
        else
            return fast_div(B, a.c_mul, a.c_shift);
    };
    const index_t pA = pixel_of(B0);
    const int jA = static_cast<int>((static_cast<uint32_t>(B0 - pA * C) + 63u) >> 6);   // <= Cw: then it is (pA + 1, 0)
    const index_t wA = pA * Cw + jA;
    index_t wB = n_words;
    if (B0 + 64 * kTailChunks < n_floats) {
        const index_t pB = pixel_of(B0 + 64 * kTailChunks);
        wB = pB * Cw + ((static_cast<uint32_t>(B0 + 64 * kTailChunks - pB * C) + 63u) >> 6);
    }
    const int count = static_cast<int>(wB - wA);   // words that start in these chunks

    const index_t avail = n_floats - B0;   // floats from the first chunk to the tensor's end: > 0
    const uint32_t* src = x + static_cast<size_t>(B0);   // wave-uniform
    uint32_t v[kTailChunks + 1];
    if (avail >= static_cast<index_t>(64 * (kTailChunks + 1))) {
#pragma unroll
        for (int k = 0; k <= kTailChunks; ++k)
            v[k] = __builtin_nontemporal_load(src + k * 64 + lane);
        // (an empty statement at the end of this branch only: without it the compiler merges the
        // two branches into one sequence of loads from 33 separately computed addresses)
        asm volatile("");
    } else {
        // the tensor ends inside these chunks: loads past the end re-read its last element
        const uint32_t last = static_cast<uint32_t>(avail) - 1;
#pragma unroll
        for (int k = 0; k <= kTailChunks; ++k)
            v[k] = src[min(static_cast<uint32_t>(k * 64 + lane), last)];
    }
    int blo = 0, bhi = 0;  // lane k: the sign bits of chunk c0 + k
    static_for<0, kTailChunks + 1>([&](auto kc) {
        constexpr int k = decltype(kc)::value;
        const uint64_t word = __builtin_amdgcn_ballot_w64(negative_bit<MODE>(v[k]));
        park_in_lane<k>(blo, bhi, static_cast<uint32_t>(word), static_cast<uint32_t>(word >> 32));
    });

    // lane l assembles word wA + l (+ 64 per further pass), in 32-bit arithmetic relative to the
    // first chunk: flat bit of pixel pA minus B0 (negative when the pixel starts before the chunk)
    // (unsigned arithmetic: the terms can approach 2^31 for rows of a billion channels, their sum
    // is below 2048)
    const uint32_t base = 0u - static_cast<uint32_t>(B0 - pA * C);
    // (every lane takes part in the lane exchange of every pass; only the store is conditional)
    for (int first = 0; first < count; first += 64) {
        const int l = first + lane;
        const int q = jA + min(l, count - 1);   // word index counted from pixel pA's first word
        const int dp = static_cast<int>(fast_div(static_cast<uint32_t>(q), a.cw_mul, a.cw_shift));
        const int j = q - dp * Cw;
        const uint32_t rel = base + static_cast<uint32_t>(dp) * static_cast<uint32_t>(C) +
                             64u * static_cast<uint32_t>(j);  // 0 <= rel < 64 * kTailChunks
        const int from = static_cast<int>(rel >> 6), off = static_cast<int>(rel & 63);
        const int len = min(64, C - 64 * j);
        const uint64_t b0 = (static_cast<uint64_t>(static_cast<uint32_t>(__shfl(bhi, from))) << 32) |
                            static_cast<uint32_t>(__shfl(blo, from));
        const uint64_t b1 = (static_cast<uint64_t>(static_cast<uint32_t>(__shfl(bhi, from + 1))) << 32) |
                            static_cast<uint32_t>(__shfl(blo, from + 1));
        uint64_t word = b0 >> off;
        if (off != 0)
            word |= b1 << (64 - off);
        if (len < 64)
            word &= (uint64_t{1} << len) - 1;  // bits past the pixel's last channel are 0
        if (l < count)
            out[wA + l] = make_uint2(static_cast<uint32_t>(word), static_cast<uint32_t>(word >> 32));
    }
}

// Fused batch-norm + shortcut + sign + bit-pack between two binary convolutions (Sec. 2.1.1 names
// the fused BN-binarization layer; Sec. 2.3's Bi-Real blocks add a real-valued shortcut first):
//   z = ((scale[c] * float(y)) + shift[c]) + r,  every operation rounded separately (no FMA),
// z optionally written out, its sign bits packed exactly as in bitpack_kernel: lane i handles
// channel 64*j + i, so y, r and z move as coalesced 256-byte runs and one ballot is one word.
// Bound by HBM: 4 (y) + 4 (r) + 4 (z) + 1/8 bytes per element.
template <bool HAS_R, bool HAS_X, bool FLAT>
__global__ __launch_bounds__(64 * kWavesPerBlock) void bn_sign_pack_kernel(
    // y, r and x_out carry no __restrict__: x_out may be r's storage, or y's (the two-kernel route
    // of dabnn_bconv2d_bn_residual stages y there); every element is read before it is written
    const int32_t* y, const float* __restrict__ scale, const float* __restrict__ shift,
    const float* r, float* x_out, uint2* __restrict__ out, int64_t n_words, int C, int Cw)
{
    const int lane = threadIdx.x & 63;
    const int wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t g0 =
        (static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave_in_block) * kWordsPerWave;
    if (g0 >= n_words)
        return;
    // z for one element; the multiply and the adds must round separately: this file is compiled
    // with -ffp-contract=off, so no v_fma_f32 / v_fmac_f32 is formed here
    auto bn = [&](int c, int yv, float rv) {
        float z = __fmul_rn(scale[c], static_cast<float>(yv));
        z = __fadd_rn(z, shift[c]);
        if (HAS_R)
            z = __fadd_rn(z, rv);
        return z;
    };
    uint32_t lo = 0, hi = 0;
    if (FLAT && g0 + kWordsPerWave <= n_words) {
        // C is a multiple of 64: word g covers the 64 consecutive elements from 64*g, and only
        // the word's position within its pixel (wave-uniform) decides the channels
        const int64_t e0 = g0 * 64 + lane;
        int yv[kWordsPerWave];
        float rv[kWordsPerWave];
#pragma unroll
        for (int k = 0; k < kWordsPerWave; ++k) {
            yv[k] = __builtin_nontemporal_load(y + e0 + k * 64);
            rv[k] = HAS_R ? __builtin_nontemporal_load(r + e0 + k * 64) : 0.0f;
        }
        int j = static_cast<int>(g0 % Cw);
        static_for<0, kWordsPerWave>([&](auto kc) {
            constexpr int k = decltype(kc)::value;
            const float z = bn(64 * j + lane, yv[k], rv[k]);
            if (HAS_X)
                __builtin_nontemporal_store(z, x_out + e0 + k * 64);
            const uint64_t word = __builtin_amdgcn_ballot_w64(static_cast<int32_t>(__float_as_uint(z)) < 0);
            if (lane == k) {
                lo = static_cast<uint32_t>(word);
                hi = static_cast<uint32_t>(word >> 32);
            }
            j = (j + 1 == Cw) ? 0 : j + 1;
        });
    } else {
        int64_t p = g0 / Cw;
        int j = static_cast<int>(g0 - p * Cw);
        static_for<0, kWordsPerWave>([&](auto kc) {
            constexpr int k = decltype(kc)::value;
            const int c = 64 * j + lane;
            bool neg = false;  // a missing channel packs as bit 0
            if (g0 + k < n_words && c < C) {
                const int64_t e = p * C + c;
                const float z = bn(c, y[e], HAS_R ? r[e] : 0.0f);
                if (HAS_X)
                    x_out[e] = z;
                neg = static_cast<int32_t>(__float_as_uint(z)) < 0;
            }
            const uint64_t word = __builtin_amdgcn_ballot_w64(neg);
            if (lane == k) {
                lo = static_cast<uint32_t>(word);
                hi = static_cast<uint32_t>(word >> 32);
            }
            if (++j == Cw) {
                j = 0;
                ++p;
            }
        });
    }
    if (lane < kWordsPerWave && g0 + lane < n_words)
        out[g0 + lane] = make_uint2(lo, hi);
}

// NHWC words -> NC1HWC2 with C2 = 128 bits (Sec. 2.1.2): one thread per 16-byte group of the
// output, so stores are fully coalesced; reads are two adjacent words of a pixel.
__global__ __launch_bounds__(256) void nc1hwc2_kernel(const uint64_t* __restrict__ in,
                                                      uint2* __restrict__ out_words, int64_t total,
                                                      int HW, int Cw, int C1, bool to_grouped)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;  // (n, c1, hw)
    if (idx >= total)
        return;
    const int hw = static_cast<int>(idx % HW);
    const int64_t t = idx / HW;
    const int c1 = static_cast<int>(t % C1);
    const int64_t n = t / C1;
    const int64_t nhwc = (n * HW + hw) * Cw + 2 * c1;  // first word of the group in NHWC order
    uint64_t* outw = reinterpret_cast<uint64_t*>(out_words);
    if (to_grouped) {
        const uint64_t w0 = in[nhwc];
        const uint64_t w1 = (2 * c1 + 1 < Cw) ? in[nhwc + 1] : 0;  // a missing second word is 0
        outw[2 * idx] = w0;
        outw[2 * idx + 1] = w1;
    } else {
        outw[nhwc] = in[2 * idx];
        if (2 * c1 + 1 < Cw)
            outw[nhwc + 1] = in[2 * idx + 1];
    }
}

}  // namespace

hipError_t launch_nc1hwc2(const uint64_t* in, uint64_t* out, int N, int H, int W, int Cw,
                          bool to_grouped, hipStream_t stream)
{
    const int C1 = (Cw + 1) / 2;
    const int64_t total = static_cast<int64_t>(N) * C1 * H * W;
    const int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffLL)
        return hipErrorInvalidValue;
    nc1hwc2_kernel<<<dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream>>>(
        in, reinterpret_cast<uint2*>(out), total, H * W, Cw, C1, to_grouped);
    return hipGetLastError();
}

hipError_t launch_bn_sign_pack(const int32_t* y, const float* scale, const float* shift,
                               const float* r, float* x_out, uint64_t* bits, int64_t n_rows, int C,
                               hipStream_t stream)
{
    const int64_t Cw = (static_cast<int64_t>(C) + 63) / 64;
    const int64_t n_words = n_rows * Cw;
    if (n_words == 0)
        return hipSuccess;
    const int64_t per_block = static_cast<int64_t>(kWordsPerWave) * kWavesPerBlock;
    const int64_t blocks = (n_words + per_block - 1) / per_block;
    if (blocks > 0x7fffffffLL)
        return hipErrorInvalidValue;
    const dim3 grid(static_cast<unsigned>(blocks)), block(64 * kWavesPerBlock);
    uint2* o = reinterpret_cast<uint2*>(bits);
    const int cw = static_cast<int>(Cw);
#define DABNN_LAUNCH(HR, HX)                                                                       \
    do {                                                                                           \
        if (C % 64 == 0)                                                                           \
            bn_sign_pack_kernel<HR, HX, true><<<grid, block, 0, stream>>>(y, scale, shift, r, x_out, \
                                                                          o, n_words, C, cw);      \
        else                                                                                       \
            bn_sign_pack_kernel<HR, HX, false><<<grid, block, 0, stream>>>(y, scale, shift, r,      \
                                                                           x_out, o, n_words, C, cw); \
    } while (0)
    if (r && x_out)
        DABNN_LAUNCH(true, true);
    else if (r)
        DABNN_LAUNCH(true, false);
    else if (x_out)
        DABNN_LAUNCH(false, true);
    else
        DABNN_LAUNCH(false, false);
#undef DABNN_LAUNCH
    return hipGetLastError();
}

hipError_t launch_bitpack(const float* x, uint64_t* out, int64_t n_rows, int C, int sign_mode,
                          hipStream_t stream)
{
    const int64_t Cw = (static_cast<int64_t>(C) + 63) / 64;
    const int64_t n_words = n_rows * Cw;
    if (n_words == 0)
        return hipSuccess;
    const int64_t per_block = static_cast<int64_t>(kWordsPerWave) * kWavesPerBlock;
    const int64_t blocks = (n_words + per_block - 1) / per_block;
    if (blocks > 0x7fffffffLL)
        return hipErrorInvalidValue;
    const dim3 grid(static_cast<unsigned>(blocks)), block(64 * kWavesPerBlock);
    const uint32_t* xi = reinterpret_cast<const uint32_t*>(x);
    uint2* o = reinterpret_cast<uint2*>(out);
    const bool flat = (C % 64) == 0;
    const int cw = static_cast<int>(Cw);
    const int tail_kernel = option(DABNN_OPT_BITPACK_ROWWISE);   // 0 by size, 1 row-wise, 2 64-bit flat stream
    if (!flat && tail_kernel != 1) {
        const int64_t n_floats = n_rows * C;
        const int64_t per_block_t = int64_t{64} * kTailChunks * kWavesPerBlock;   // elements per workgroup
        const int64_t blocks_t = (n_floats + per_block_t - 1) / per_block_t;
        if (blocks_t > 0x7fffffffLL)
            return hipErrorInvalidValue;
        const dim3 grid_t(static_cast<unsigned>(blocks_t));
        TailArgs args{n_words, n_floats, C, cw, 0, 0, 0, 0};
        division_constants(static_cast<uint32_t>(C), args.c_mul, args.c_shift);
        division_constants(static_cast<uint32_t>(cw), args.cw_mul, args.cw_shift);
        // 32-bit indices: the element count, rounded up to whole workgroups, below 2^32
        const bool wide = tail_kernel == 2 || n_floats >= (int64_t{1} << 31);
#define DABNN_LAUNCH(MODE, WIDE) bitpack_tail_kernel<MODE, WIDE><<<grid_t, block, 0, stream>>>(xi, o, args)
        if (sign_mode == 0) {
            if (wide)
                DABNN_LAUNCH(0, true);
            else
                DABNN_LAUNCH(0, false);
        } else {
            if (wide)
                DABNN_LAUNCH(1, true);
            else
                DABNN_LAUNCH(1, false);
        }
#undef DABNN_LAUNCH
        return hipGetLastError();
    }
    if (sign_mode == 0) {
        if (flat)
            bitpack_kernel<0, true><<<grid, block, 0, stream>>>(xi, o, n_words, C, cw);
        else
            bitpack_kernel<0, false><<<grid, block, 0, stream>>>(xi, o, n_words, C, cw);
    } else {
        if (flat)
            bitpack_kernel<1, true><<<grid, block, 0, stream>>>(xi, o, n_words, C, cw);
        else
            bitpack_kernel<1, false><<<grid, block, 0, stream>>>(xi, o, n_words, C, cw);
    }
    return hipGetLastError();
}

}  // namespace dabnn

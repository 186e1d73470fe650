// Binary 3x3 convolution on the int8 matrix cores, fed from the PACKED bits (Sec. 2.1.2, Eq. 6-7
// give the result; this file computes the same integers as a matrix product).
//
// With a = 1 for an activation of -1 (0 for +1) and s = +1 / -1 for a weight of +1 / -1,
//     y = sum_k (1 - 2 a_k) s_k = S - 2 * sum_k a_k s_k,      S = sum_k s_k = K - 2 popcount(w),
// so the convolution is one int8 product of 0/1 activations with +-1 weights plus a constant per
// output channel; an out-of-image tap is a = 0 (+1), which is the all-zero word the packed tensor
// already stands for.  The matrix instruction contracts 32 products whose order is free as long
// as both operands agree on it, which makes the expansion of the activation bits cheap:
//   lane (pixel m, half h) of a wavefront holds one 32-bit word x of the pixel's window;
//   step j in {0, 1} of that word uses xs = x >> 4j, and operand register v in 0..3 is
//   xs & (0x01010101 << v): byte b holds bit 4j + v + 8b of x, as the value 2^v.
// One AND per operand register.  The weights are prepared once per model in exactly that order
// (dabnn_prepare_weights_mfma): byte (h, v, b) of a step is -s * 2^(3 - v), so every product is
// -+8 a; the accumulators start at 4 S and end at 4 S - 8 sum a s = 4 y: one shift per output.
//
// FP4 mode (v_mfma_scale_f32_32x32x64_f8f6f4 with both operands in the 4-bit E2M1 format, scales
// 1.0): twice the products per instruction.  One 32-bit word x per lane is one whole operand: the
// registers are x & 0x11111111 (bit 4k as the value 0.5 in nibble k), x & 0x22222222 (bit 4k+1 as
// 1.0), x & 0x44444444 (bit 4k+2 as 2.0) and (x >> 3) & 0x11111111 (bit 4k+3 as 0.5); the prepared
// weights are -s * 4, -s * 2, -s * 1, -s * 4 in the same places, so every product is -+2 a exactly
// and the fp32 accumulators, which start at S, end at the integer S - 2 sum a s = y.
//
//   mfma_prepare_weights_kernel : packed filters -> [Cout/32][steps][64 lanes][16 B], S[Cout]
//   bconv_mfma_bits_kernel      : a wavefront owns 32*MB pixels x 32*NB channels (MB x NB
//       v_mfma_i32_32x32x32_i8 accumulators); the four wavefronts of a workgroup own different
//       pixels and the same channels, and share the weight operands through LDS (double-buffered
//       stages of CH steps, one barrier per stage); the activation words come straight from the
//       packed tensor (a few KB per tile, cache-resident) one stage ahead.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

#include "kernel_util.h"   // fast_div, division_constants
#include "launch.h"

namespace dabnn {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));

// Order of the K dimension, shared by the two kernels.  A pixel's tap holds 2*CW dwords.  They are
// consumed in R rounds of 2*W dwords; in a round the lanes of half h take dwords 2W*r + W*h + q,
// q < W, and every dword feeds two steps (j = 0, 1).  Step index t = ((tap*R + r)*W + q)*2 + j.
__host__ __device__ constexpr int mfma_w(int cw) { return cw < 4 ? cw : 4; }

// One thread per (output channel, step, half, register): 4 bytes out.
template <bool FP4>
__global__ __launch_bounds__(256) void mfma_prepare_weights_kernel(
    const uint32_t* __restrict__ wp, int8_t* __restrict__ wq, int32_t* __restrict__ sw, int Cout,
    int Cw, int steps)
{
    const int W = mfma_w(Cw), R = Cw / W, D = 2 * Cw;
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t total = static_cast<int64_t>(Cout) * steps * 8;
    if (idx < total) {
        const int v = static_cast<int>(idx & 3);
        const int h = static_cast<int>((idx >> 2) & 1);
        const int64_t ct = idx >> 3;
        const int t = static_cast<int>(ct % steps);
        const int n = static_cast<int>(ct / steps);
        const int j = FP4 ? 0 : (t & 1);
        const int u = FP4 ? t : (t >> 1);  // (tap*R + r)*W + q
        const int q = u % W;
        const int r = (u / W) % R;
        const int tap = u / (W * R);
        const uint32_t x = wp[(static_cast<int64_t>(n) * 9 + tap) * D + 2 * W * r + W * h + q];
        uint32_t out = 0;
        if (FP4) {
            // -2 s / (the activation bit's value 0.5, 1, 2, 0.5) in E2M1: 1.0 = 0010, 2.0 = 0100,
            // 4.0 = 0110, sign = 1000
            const uint32_t magnitude = v == 1 ? 0x4u : (v == 2 ? 0x2u : 0x6u);
            for (int k = 0; k < 8; ++k) {
                const uint32_t bit = (x >> (4 * k + v)) & 1u;
                out |= (magnitude | (bit ? 0u : 0x8u)) << (4 * k);
            }
        } else {
            // -8 s / (the activation bit's value 2^v)
            for (int b = 0; b < 4; ++b) {
                const uint32_t bit = (x >> (4 * j + v + 8 * b)) & 1u;
                const int val = (bit ? 1 : -1) * (8 >> v);
                out |= (static_cast<uint32_t>(val) & 0xffu) << (8 * b);
            }
        }
        // [n/32][t][lane = 32h + n%32][16 bytes = 4 registers]
        const int64_t o = ((static_cast<int64_t>(n >> 5) * steps + t) * 64 + 32 * h + (n & 31)) * 16 + 4 * v;
        *reinterpret_cast<uint32_t*>(wq + o) = out;
    }
    // S[n] = K - 2 * popcount of the filter's words (Cin % 64 == 0: no padding bits)
    if (idx < Cout) {
        const int n = static_cast<int>(idx);
        int pop = 0;
        for (int d = 0; d < 9 * D; ++d)
            pop += __popc(wp[static_cast<int64_t>(n) * 9 * D + d]);
        sw[n] = 9 * 64 * Cw - 2 * pop;
    }
}

struct MfmaArgs {
    int H, W, Ho, Wo, pad, Cout, total_pix;
    uint32_t hw, hw_mul, hw_shift;   // Ho*Wo and its multiply-shift division constants
    uint32_t wo_mul, wo_shift;       // those of Wo
};

template <int CW, int MB, int NB, bool FP4>
struct MfmaGeom {
    static constexpr int W = mfma_w(CW);
    static constexpr int R = CW / W;
    static constexpr int D = 2 * CW;
    static constexpr int SPD = FP4 ? 1 : 2;            // matrix instructions (steps) per dword
    static constexpr int STEPS = 9 * CW * SPD;
    // (tap, round) pairs of W dwords per LDS stage: a window row at one word per pixel, otherwise
    // one pair (larger stages, i.e. fewer barriers, measured no faster)
    static constexpr int GROUPS = CW == 1 ? 3 : 1;
    static constexpr int UPS = GROUPS * W;             // dwords a lane consumes per stage
    static constexpr int CH = UPS * SPD;               // steps per stage
    static constexpr int STAGES = STEPS / CH;
    static constexpr int STAGE_BYTES = CH * NB * 1024;
    static constexpr int PIECES = STAGE_BYTES / 16;    // 16-byte copies per stage
    static constexpr int UNITS = (PIECES + 255) / 256; // ... per thread (the last one may be partial)
    static_assert(STEPS % CH == 0 && PIECES % 64 == 0 && (9 * R) % GROUPS == 0, "stage geometry");
};

// MASKED = false: the tensor has at least 32*MB pixels, and a wavefront whose tile would reach
// past the end computes the LAST 32*MB pixels instead (some of them a second time, with the same
// results), so that no load or store needs a bounds check.  MASKED = true: fewer pixels than one
// tile; rows past the end repeat the last pixel and are not stored.
//
// BITS = true: the fused threshold epilogue of dabnn_bconv2d_bnsign.  Instead of y the kernel
// writes the next layer's packed activations: bit c of a pixel is (y < thr[c]) XOR flip bit c.  A
// lane holds one channel of 16 pixels, so one compare per accumulator register gives a wave-wide
// mask whose two halves are 32 consecutive channels of two pixels: half a packed word each, which
// lane 0 and lane 32 store.
template <int CW, int S, int MB, int NB, bool MASKED, bool FP4, bool BITS>
__global__ __launch_bounds__(256) void bconv_mfma_bits_kernel(const uint32_t* __restrict__ a,
                                                              const int8_t* __restrict__ wq,
                                                              const int32_t* __restrict__ sw,
                                                              int32_t* __restrict__ y,
                                                              const int32_t* __restrict__ thr,
                                                              const uint32_t* __restrict__ flip32,
                                                              const MfmaArgs p)
{
    using G = MfmaGeom<CW, MB, NB, FP4>;
    __shared__ __attribute__((aligned(16))) int8_t lds_b[2][G::STAGE_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = lane & 31, h = lane >> 5;
    int pix0 = (blockIdx.x * 4 + wave) * (32 * MB);   // first pixel of this wavefront
    if (!MASKED)
        pix0 = min(pix0, p.total_pix - 32 * MB);
    const int nblk0 = blockIdx.y * NB;                       // first 32-channel block

    // Per pixel block: dword offset of the window's top-left tap (may lie outside the tensor; used
    // only for taps inside the image) and one validity bit per tap.
    int a_base[MB];
    uint32_t a_valid[MB];
#pragma unroll
    for (int i = 0; i < MB; ++i) {
        const int pc = min(pix0 + 32 * i + m, p.total_pix - 1);  // rows past the end repeat
        const int n = static_cast<int>(fast_div(static_cast<uint32_t>(pc), p.hw_mul, p.hw_shift));
        const int rem = pc - n * static_cast<int>(p.hw);
        const int ho = static_cast<int>(fast_div(static_cast<uint32_t>(rem), p.wo_mul, p.wo_shift));
        const int hi0 = ho * S - p.pad;
        const int wi0 = (rem - ho * p.Wo) * S - p.pad;
        a_base[i] = ((n * p.H + hi0) * p.W + wi0) * G::D + G::W * h;
        // bit 3 ti + tj: row hi0 + ti and column wi0 + tj inside the image
        uint32_t rows = 0, cols = 0;
#pragma unroll
        for (int t = 0; t < 3; ++t) {
            rows |= (static_cast<unsigned>(hi0 + t) < static_cast<unsigned>(p.H) ? 1u : 0u) << (3 * t);
            cols |= (static_cast<unsigned>(wi0 + t) < static_cast<unsigned>(p.W) ? 1u : 0u) << t;
        }
        a_valid[i] = (rows * 7u) & (cols * 0x49u);
    }

    // The activation dwords of stage st for this lane: raw[i][k], k < UPS.  A tap outside the image
    // reads offset 0 and is cleared: both through an all-ones / all-zeros lane value, so that no
    // condition travels through a scalar register pair.
    auto load_a = [&](int st, uint32_t (&raw)[MB][G::UPS]) {
        // the stage is GROUPS consecutive (tap, round) pairs of W dwords each
#pragma unroll
        for (int g = 0; g < G::GROUPS; ++g) {
            const int tr = st * G::GROUPS + g;
            const int tap = tr / G::R, r = tr - tap * G::R;
            const int ti = tap / 3, tj = tap - 3 * ti;
            const int tap_off = (ti * p.W + tj) * G::D + 2 * G::W * r;
#pragma unroll
            for (int i = 0; i < MB; ++i) {
                const uint32_t keep = static_cast<uint32_t>(-static_cast<int>((a_valid[i] >> tap) & 1u));
                const uint32_t off = static_cast<uint32_t>(a_base[i] + tap_off) & keep;
                if constexpr (G::W == 4) {
                    const uint4 x = *reinterpret_cast<const uint4*>(a + off);
                    raw[i][4 * g + 0] = x.x & keep;
                    raw[i][4 * g + 1] = x.y & keep;
                    raw[i][4 * g + 2] = x.z & keep;
                    raw[i][4 * g + 3] = x.w & keep;
                } else if constexpr (G::W == 2) {
                    const uint2 x = *reinterpret_cast<const uint2*>(a + off);
                    raw[i][2 * g + 0] = x.x & keep;
                    raw[i][2 * g + 1] = x.y & keep;
                } else {
                    raw[i][g] = a[off] & keep;
                }
            }
        }
    };

    // Weight stage st of channel block nb: CH KB contiguous at ((nblk0 + nb)*STEPS + st*CH) KB.
    // Thread tid copies UNITS 16-byte pieces; piece index c = tid + 256*k over [nb][CH*64 lanes].
    auto load_b = [&](int st, v4i (&stage)[G::UNITS]) {
#pragma unroll
        for (int k = 0; k < G::UNITS; ++k) {
            const int c = tid + 256 * k;
            if (256 * (k + 1) > G::PIECES && c >= G::PIECES)   // partial last unit (whole wavefronts)
                continue;
            const int nb = c / (G::CH * 64), rest = c % (G::CH * 64);
            const int8_t* src = wq + ((static_cast<int64_t>(nblk0 + nb) * G::STEPS + st * G::CH) * 64 + rest) * 16;
            stage[k] = *reinterpret_cast<const v4i*>(src);
        }
    };
    auto store_b = [&](int buf, const v4i (&stage)[G::UNITS]) {
#pragma unroll
        for (int k = 0; k < G::UNITS; ++k)
            if (256 * (k + 1) <= G::PIECES || tid + 256 * k < G::PIECES)
                *reinterpret_cast<v4i*>(&lds_b[buf][(tid + 256 * k) * 16]) = stage[k];
    };

    // every accumulator register of a lane belongs to one output channel: they start at that
    // channel's constant (4 S for int8, S for FP4) and the matrix instructions subtract from it
    using acc_t = std::conditional_t<FP4, v16f, v16i>;
    acc_t acc[MB][NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int s_w = sw[(nblk0 + nb) * 32 + m];
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                if constexpr (FP4)
                    acc[i][nb][v] = static_cast<float>(s_w);
                else
                    acc[i][nb][v] = 4 * s_w;
            }
    }

    uint32_t raw[MB][G::UPS], raw_next[MB][G::UPS];
    v4i stage[G::UNITS];
    load_a(0, raw);
    load_b(0, stage);
    store_b(0, stage);
    __syncthreads();

#pragma unroll
    for (int st = 0; st < G::STAGES; ++st) {
        const int buf = st & 1;
        if (st + 1 < G::STAGES) {
            load_b(st + 1, stage);   // requested before the stage's arithmetic, consumed after it
            load_a(st + 1, raw_next);
        }
#pragma unroll
        for (int c = 0; c < G::CH; ++c) {
            const int k = c / G::SPD, j = c % G::SPD;
            v4i bf[NB];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                bf[nb] = *reinterpret_cast<const v4i*>(&lds_b[buf][((nb * G::CH + c) * 64 + lane) * 16]);
#pragma unroll
            for (int i = 0; i < MB; ++i) {
                if constexpr (FP4) {
                    const uint32_t x = raw[i][k];
                    const v8i af = {static_cast<int>(x & 0x11111111u), static_cast<int>(x & 0x22222222u),
                                    static_cast<int>(x & 0x44444444u), static_cast<int>((x >> 3) & 0x11111111u),
                                    0, 0, 0, 0};
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        const v8i b8 = {bf[nb].x, bf[nb].y, bf[nb].z, bf[nb].w, 0, 0, 0, 0};
                        // formats 4 = FP4 (E2M1) for both operands; scales 127 = 2^0
                        acc[i][nb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(af, b8, acc[i][nb], 4, 4, 0, 127, 0, 127);
                    }
                } else {
                    const uint32_t xs = j ? (raw[i][k] >> 4) : raw[i][k];
                    v4i af;
                    af.x = static_cast<int>(xs & 0x01010101u);
                    af.y = static_cast<int>(xs & 0x02020202u);
                    af.z = static_cast<int>(xs & 0x04040404u);
                    af.w = static_cast<int>(xs & 0x08080808u);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        acc[i][nb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af, bf[nb], acc[i][nb], 0, 0, 0);
                }
            }
        }
        // With the fused epilogue (and with the masked stores of the tiny-input variant) the
        // compiler otherwise moves the matrix instructions past all later stages, towards the
        // compares that use their results, and keeps every operand of the whole K loop alive: an
        // empty statement that "uses" the accumulators keeps the instructions of a stage inside
        // the stage.
        if constexpr (BITS || MASKED) {
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    asm volatile("" : "+a"(acc[i][nb]));   // the stage's results exist here, in AGPRs
        }
        if (st + 1 < G::STAGES) {
            // buffer buf^1 was last read in stage st-1, which every wavefront has left (barrier)
            store_b(buf ^ 1, stage);
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int k = 0; k < G::UPS; ++k)
                    raw[i][k] = raw_next[i][k];
        }
        __syncthreads();
    }

    // Accumulator register v of lane l is C[8*(v/4) + 4*(l/32) + v%4][l%32]: lanes 0..31 of one
    // store instruction write 32 consecutive channels (128 bytes) of one pixel.
    // A row of the tile is a wave-uniform address (scalar arithmetic) plus one per-lane offset
    // that never changes: channel and the 4h rows of the upper half-wave.
    auto output = [&](const acc_t& c, int v) -> int {
        if constexpr (FP4)
            return static_cast<int>(c[v]);   // an integer below 2^24: exact
        else
            return c[v] >> 2;                // a multiple of 4
    };
    int rows_left = p.total_pix - pix0 - 4 * h;   // MASKED: this lane stores rows below that
    if constexpr (BITS) {
        // the packed output as 32-bit halves: [pixel][Cout/32]
        uint32_t* out32 = reinterpret_cast<uint32_t*>(y);
        const int halves = p.Cout >> 5;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int co = (nblk0 + nb) * 32 + m;
            int t = thr[co];
            const bool fl = (flip32[nblk0 + nb] >> m) & 1u;
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = 32 * i + 8 * (v / 4) + (v & 3) + 4 * h;
                    asm volatile("" : "+v"(t));   // one compare at a time: no 64 masks computed ahead
                    const uint64_t mask = __builtin_amdgcn_ballot_w64((output(acc[i][nb], v) < t) != fl);
                    const uint32_t word = h ? static_cast<uint32_t>(mask >> 32) : static_cast<uint32_t>(mask);
                    if (m == 0 && (!MASKED || row < p.total_pix - pix0))
                        out32[static_cast<size_t>(pix0 + row) * halves + (nblk0 + nb)] = word;
                }
        }
    } else {
    char* ybase = reinterpret_cast<char*>(y) + static_cast<size_t>(pix0) * p.Cout * 4;
    const size_t row_bytes = static_cast<size_t>(p.Cout) * 4;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int co = (nblk0 + nb) * 32 + m;
        const uint32_t lane_off = (static_cast<uint32_t>(4 * h) * p.Cout + co) * 4u;
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = 32 * i + 8 * (v / 4) + (v & 3);   // + 4h, in lane_off
                const int out = output(acc[i][nb], v);
                char* row_ptr = ybase + row * row_bytes;
                if constexpr (MASKED)
                    asm volatile("" : "+v"(rows_left));  // one compare at a time: no hoisted masks
                if (!MASKED || row < rows_left)
                    __builtin_nontemporal_store(out, reinterpret_cast<int*>(row_ptr + lane_off));
            }
    }
    }
}

template <int CW, int S, int MB, int NB, bool FP4, bool BITS>
hipError_t launch_mfma_bits_inst(const uint32_t* a, const int8_t* wq, const int32_t* sw, int32_t* y,
                                 const int32_t* thr, const uint32_t* flip32, const ConvShape& s,
                                 hipStream_t stream)
{
    const int64_t total_pix = static_cast<int64_t>(s.N) * s.Ho * s.Wo;
    const int64_t tiles = (total_pix + 128 * MB - 1) / (128 * MB);
    if (tiles > 0x7fffffff)
        return hipErrorNotSupported;
    MfmaArgs p{s.H, s.W, s.Ho, s.Wo, s.pad, s.Cout, static_cast<int>(total_pix), 0, 0, 0, 0, 0};
    p.hw = static_cast<uint32_t>(s.Ho) * static_cast<uint32_t>(s.Wo);
    division_constants(p.hw, p.hw_mul, p.hw_shift);
    division_constants(static_cast<uint32_t>(s.Wo), p.wo_mul, p.wo_shift);
    const dim3 grid(static_cast<unsigned>(tiles), static_cast<unsigned>(s.Cout / (32 * NB)));
    if (total_pix >= 32 * MB)
        bconv_mfma_bits_kernel<CW, S, MB, NB, false, FP4, BITS><<<grid, dim3(256), 0, stream>>>(a, wq, sw, y, thr, flip32, p);
    else
        bconv_mfma_bits_kernel<CW, S, MB, NB, true, FP4, BITS><<<grid, dim3(256), 0, stream>>>(a, wq, sw, y, thr, flip32, p);
    return hipGetLastError();
}

template <int CW, int S, bool FP4>
hipError_t launch_mfma_bits_cw(const uint32_t* a, const int8_t* wq, const int32_t* sw, int32_t* y,
                               const int32_t* thr, const uint32_t* flip32, const ConvShape& s,
                               hipStream_t stream)
{
    // 64 pixels x 64 channels per wavefront (three or four workgroups resident per CU).  When the
    // number of such workgroup tiles lies just above three per CU, the launch would end in a
    // nearly empty second round; wavefronts of 128 pixels halve the tile count and everything is
    // resident at once (measured at batch 256, int8: 14x14x256->256 26.5 us against 29.3).
    const int64_t total_pix = static_cast<int64_t>(s.N) * s.Ho * s.Wo;
    const int64_t small_tiles = ((total_pix + 255) / 256) * (s.Cout / 64);
    const int64_t cus = device_cu_count();
    const int mb = option(DABNN_OPT_MFMA_PIXEL_BLOCKS);
    const bool big = mb == 4 || (mb == 0 && small_tiles > 3 * cus && small_tiles <= 4 * cus);
    if (thr != nullptr) {   // fused threshold epilogue: packed words instead of y
        if (big)
            return launch_mfma_bits_inst<CW, S, 4, 2, FP4, true>(a, wq, sw, y, thr, flip32, s, stream);
        return launch_mfma_bits_inst<CW, S, 2, 2, FP4, true>(a, wq, sw, y, thr, flip32, s, stream);
    }
    if (big)
        return launch_mfma_bits_inst<CW, S, 4, 2, FP4, false>(a, wq, sw, y, thr, flip32, s, stream);
    return launch_mfma_bits_inst<CW, S, 2, 2, FP4, false>(a, wq, sw, y, thr, flip32, s, stream);
}

}  // namespace

bool bconv_mfma_bits_supports(const ConvShape& s)
{
    // whole words (no padding bits inside K), 64-channel tiles, 32-bit dword offsets into the
    // packed activations, 32-bit pixel indices up to a rounded-up grid, and 32-bit byte offsets
    // inside an output tile
    const int64_t act_dwords = static_cast<int64_t>(s.N) * s.H * s.W * s.Cw * 2;
    const int64_t total_pix = static_cast<int64_t>(s.N) * s.Ho * s.Wo;
    return s.kh == 3 && s.kw == 3 && (s.stride == 1 || s.stride == 2) && s.Cin % 64 == 0 &&
           (s.Cw == 1 || s.Cw == 2 || s.Cw == 4 || s.Cw == 8) && s.Cout % 64 == 0 &&
           act_dwords < (int64_t{1} << 31) && total_pix < (int64_t{1} << 31) - 4096 && s.Cout <= 8192;
}

// Operand bytes of the prepared filters: one byte (int8) or one nibble (FP4) per weight.
static size_t mfma_operand_bytes(const ConvShape& s, int format)
{
    const size_t weights = static_cast<size_t>(s.Cout) * 9 * 64 * s.Cw;
    return format == 1 ? weights / 2 : weights;
}

size_t mfma_weights_bytes(const ConvShape& s, int format)
{
    return mfma_operand_bytes(s, format) + static_cast<size_t>(s.Cout) * 4;
}

hipError_t launch_prepare_weights_mfma(const uint64_t* w, void* wq, const ConvShape& s, int format,
                                       hipStream_t stream)
{
    if (!bconv_mfma_bits_supports(s) || (format != 0 && format != 1))
        return hipErrorNotSupported;
    const int steps = (format == 1 ? 9 : 18) * s.Cw;
    const int64_t total = static_cast<int64_t>(s.Cout) * steps * 8;
    int8_t* q = static_cast<int8_t*>(wq);
    int32_t* sw = reinterpret_cast<int32_t*>(q + mfma_operand_bytes(s, format));
    const dim3 grid(static_cast<unsigned>((total + 255) / 256)), block(256);
    const uint32_t* w32 = reinterpret_cast<const uint32_t*>(w);
    if (format == 1)
        mfma_prepare_weights_kernel<true><<<grid, block, 0, stream>>>(w32, q, sw, s.Cout, s.Cw, steps);
    else
        mfma_prepare_weights_kernel<false><<<grid, block, 0, stream>>>(w32, q, sw, s.Cout, s.Cw, steps);
    return hipGetLastError();
}

hipError_t launch_bconv_mfma_bits(const uint64_t* a, const void* wq, int32_t* y, const int32_t* thr,
                                  const uint64_t* flip, const ConvShape& s, int format,
                                  hipStream_t stream)
{
    if (!bconv_mfma_bits_supports(s) || (format != 0 && format != 1))
        return hipErrorNotSupported;
    const uint32_t* a32 = reinterpret_cast<const uint32_t*>(a);
    const int8_t* q = static_cast<const int8_t*>(wq);
    const int32_t* sw = reinterpret_cast<const int32_t*>(q + mfma_operand_bytes(s, format));
    const uint32_t* f32 = reinterpret_cast<const uint32_t*>(flip);
#define DABNN_CASE(CW, S)                                                        \
    return format == 1 ? launch_mfma_bits_cw<CW, S, true>(a32, q, sw, y, thr, f32, s, stream) \
                       : launch_mfma_bits_cw<CW, S, false>(a32, q, sw, y, thr, f32, s, stream)
    switch (s.Cw * 2 + (s.stride == 2 ? 1 : 0)) {
        case 2: DABNN_CASE(1, 1);
        case 3: DABNN_CASE(1, 2);
        case 4: DABNN_CASE(2, 1);
        case 5: DABNN_CASE(2, 2);
        case 8: DABNN_CASE(4, 1);
        case 9: DABNN_CASE(4, 2);
        case 16: DABNN_CASE(8, 1);
        case 17: DABNN_CASE(8, 2);
        default: return hipErrorNotSupported;
    }
#undef DABNN_CASE
}

}  // namespace dabnn

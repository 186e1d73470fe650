// Binary direct convolution (Sec. 2.1.2, Eq. 6-7) for gfx950 wave64.
//
//   y[n,ho,wo,co] = K - 2 * sum over taps and words of popcount(a XOR w)
//
// The paper's point is the loop order: keep one output's popcounts in a register and reduce
// once at the end (Eq. 6-7), and lay memory out so that a sliding 3x3 window reuses what is
// already in registers (NC1HWC2, Fig. 3).  On gfx950 v_bcnt_u32_b32 adds the popcount into an
// accumulator directly, so the whole inner step is v_xor_b32 + v_bcnt_u32_b32 per 32 bits and
// there is no horizontal reduction at all.  What remains is feeding those two instructions.
//
// Kernel families in this file:
//   reference : one thread per output, bounds-checked, any shape.
//   wreg      : "weight-stationary".  Lane l of a wavefront owns output channel 64*g + l and
//               keeps that filter's 9*Cw packed words in VGPRs for the wavefront's lifetime.
//               The activation word of a tap is the same for all 64 lanes, so it is fetched
//               with scalar loads and used as the SGPR operand of v_xor_b32: no LDS, no
//               vector-memory traffic in the loop, and NHWC stores that are 256 contiguous
//               bytes per pixel.  A wavefront walks P output pixels of one row at a time and
//               loads each input column of the (P-1)*stride+3 wide window once per kernel row,
//               which is the paper's window reuse with SGPRs in place of NEON registers.
#include "kernel_util.h"
#include "launch.h"

namespace dabnn {
namespace {

// ------------------------------------------------------------------------------ reference

__global__ __launch_bounds__(256) void bconv_reference_kernel(
    const uint64_t* __restrict__ a, const uint64_t* __restrict__ w, int32_t* __restrict__ y,
    ConvShape s, int64_t total)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (idx >= total)
        return;
    const int co = static_cast<int>(idx % s.Cout);
    int64_t pix = idx / s.Cout;
    const int wo = static_cast<int>(pix % s.Wo);
    pix /= s.Wo;
    const int ho = static_cast<int>(pix % s.Ho);
    const int n = static_cast<int>(pix / s.Ho);

    int diff = 0;
    for (int i = 0; i < s.kh; ++i) {
        const int hi = ho * s.stride - s.pad + i;
        for (int j = 0; j < s.kw; ++j) {
            const int wi = wo * s.stride - s.pad + j;
            const uint64_t* wp = w + ((static_cast<int64_t>(co) * s.kh + i) * s.kw + j) * s.Cw;
            if (hi >= 0 && hi < s.H && wi >= 0 && wi < s.W) {
                const uint64_t* ap = a + ((static_cast<int64_t>(n) * s.H + hi) * s.W + wi) * s.Cw;
                for (int q = 0; q < s.Cw; ++q)
                    diff += __popcll(ap[q] ^ wp[q]);
            } else {
                for (int q = 0; q < s.Cw; ++q)  // outside the image: every activation bit is 0
                    diff += __popcll(wp[q]);
            }
        }
    }
    y[idx] = s.K - 2 * diff;
}

// One thread per (pixel, 64-channel output word) of the fused conv + threshold + bit-pack.
__global__ __launch_bounds__(256) void bconv_bnsign_reference_kernel(
    const uint64_t* __restrict__ a, const uint64_t* __restrict__ w,
    const int32_t* __restrict__ thr, const uint64_t* __restrict__ flip, uint64_t* __restrict__ out,
    ConvShape s, int64_t total)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (idx >= total)
        return;
    const int words = (s.Cout + 63) / 64;
    const int word = static_cast<int>(idx % words);
    int64_t pix = idx / words;
    const int wo = static_cast<int>(pix % s.Wo);
    pix /= s.Wo;
    const int ho = static_cast<int>(pix % s.Ho);
    const int n = static_cast<int>(pix / s.Ho);
    uint64_t bits = 0;
    for (int c = 0; c < 64 && word * 64 + c < s.Cout; ++c) {
        const int co = word * 64 + c;
        int diff = 0;
        for (int i = 0; i < s.kh; ++i) {
            const int hi = ho * s.stride - s.pad + i;
            for (int j = 0; j < s.kw; ++j) {
                const int wi = wo * s.stride - s.pad + j;
                const uint64_t* wp = w + ((static_cast<int64_t>(co) * s.kh + i) * s.kw + j) * s.Cw;
                const bool inside = hi >= 0 && hi < s.H && wi >= 0 && wi < s.W;
                const uint64_t* ap = a + ((static_cast<int64_t>(n) * s.H + (inside ? hi : 0)) * s.W +
                                          (inside ? wi : 0)) * s.Cw;
                for (int q = 0; q < s.Cw; ++q)
                    diff += __popcll((inside ? ap[q] : 0ull) ^ wp[q]);
            }
        }
        const int yv = s.K - 2 * diff;
        if (yv < thr[co])
            bits |= 1ull << c;
    }
    out[idx] = bits ^ flip[word];
}

// ------------------------------------------------------------------------------ wreg

// A packed pixel of zeros (= every channel +1): what a tap outside the image reads.  Never
// written; it is not const-qualified only so that it lives in the same (global) address space as
// the activation tensor and a select between the two stays a scalar load.
__device__ uint32_t g_zero_pixel[16];

// acc += sum_d popcount(a[d] ^ w[d]): the inner step of Eq. 6 for NP x 32 bits of one output.
// Every a[d] is wave-uniform and sits in an SGPR (the scalar operand of v_xor_b32).  Written as
// assembly so that the accumulation stays one v_bcnt chain per output (the compiler otherwise
// re-associates it into extra adds), several pairs per statement so that no padding is
// inserted between statements.
#define DABNN_XP(A, W) "v_xor_b32 %1, %" #A ", %" #W "\n\tv_bcnt_u32_b32 %0, %1, %0\n\t"
template <int NP>
struct XorPopc;
template <>
struct XorPopc<2> {
    static __device__ __forceinline__ void run(int& acc, const uint32_t* a, const uint32_t* w)
    {
        uint32_t t;
        asm(DABNN_XP(2, 4) DABNN_XP(3, 5)
            : "+v"(acc), "=&v"(t)
            : "s"(a[0]), "s"(a[1]), "v"(w[0]), "v"(w[1]));
    }
};
template <>
struct XorPopc<4> {
    static __device__ __forceinline__ void run(int& acc, const uint32_t* a, const uint32_t* w)
    {
        uint32_t t;
        asm(DABNN_XP(2, 6) DABNN_XP(3, 7) DABNN_XP(4, 8) DABNN_XP(5, 9)
            : "+v"(acc), "=&v"(t)
            : "s"(a[0]), "s"(a[1]), "s"(a[2]), "s"(a[3]), "v"(w[0]), "v"(w[1]), "v"(w[2]), "v"(w[3]));
    }
};
template <>
struct XorPopc<8> {
    static __device__ __forceinline__ void run(int& acc, const uint32_t* a, const uint32_t* w)
    {
        uint32_t t;
        asm(DABNN_XP(2, 10) DABNN_XP(3, 11) DABNN_XP(4, 12) DABNN_XP(5, 13) DABNN_XP(6, 14)
                DABNN_XP(7, 15) DABNN_XP(8, 16) DABNN_XP(9, 17)
            : "+v"(acc), "=&v"(t)
            : "s"(a[0]), "s"(a[1]), "s"(a[2]), "s"(a[3]), "s"(a[4]), "s"(a[5]), "s"(a[6]), "s"(a[7]),
              "v"(w[0]), "v"(w[1]), "v"(w[2]), "v"(w[3]), "v"(w[4]), "v"(w[5]), "v"(w[6]), "v"(w[7]));
    }
};
#undef DABNN_XP

// D dwords of one (input column, output pixel, kernel tap) in statements of at most 8 pairs.
template <int D>
__device__ __forceinline__ void xor_popc_acc(int& acc, const uint32_t* a, const uint32_t* w)
{
    constexpr int NP = D < 8 ? D : 8;
#pragma unroll
    for (int d = 0; d < D; d += NP)
        XorPopc<NP>::run(acc, a + d, w + d);
}

// Geometry of one task = P consecutive output pixels of one output row, for 64 output channels.
// The 3 x WIN input window under the task is consumed in "units" of UC columns (16 dwords), the
// granularity of the scalar-load software pipeline.
template <int CW, int S, int P>
struct WregGeom {
    static constexpr int D = 2 * CW;              // dwords per packed pixel
    static constexpr int KD = 9 * D;              // dwords per packed filter
    static constexpr int WIN = (P - 1) * S + 3;   // input columns under P adjacent outputs
    static constexpr int UC = (CW >= 8) ? 1 : 8 / CW;
    static constexpr int UPR = (WIN + UC - 1) / UC;  // units per kernel row
    static constexpr int U = 3 * UPR;
    static constexpr int UD = UC * D;             // dwords per unit
};

struct TaskPos {
    int n, ho, chunk;
};

template <int CW, int S, int P, int UNIT, int UD>
__device__ __forceinline__ void wreg_load_unit(uint32_t (&buf)[UD], const uint32_t* __restrict__ a,
                                               const TaskPos& tp, int H, int W, int pad)
{
    using G = WregGeom<CW, S, P>;
    static_assert(UD == G::UD, "unit buffer size");
    constexpr int i = UNIT / G::UPR;
    constexpr int c0 = (UNIT % G::UPR) * G::UC;
    const int hi = tp.ho * S - pad + i;
    const bool rv = static_cast<unsigned>(hi) < static_cast<unsigned>(H);
    const uint32_t* rowp = a + (static_cast<size_t>(tp.n) * H + (rv ? hi : 0)) * W * G::D;
    const int wi0 = tp.chunk * (P * S) - pad + c0;
#pragma unroll
    for (int cc = 0; cc < G::UC; ++cc) {
        if (c0 + cc < G::WIN) {
            const int wi = wi0 + cc;
            const bool v = rv && static_cast<unsigned>(wi) < static_cast<unsigned>(W);
            // Outside the image the tap is an all-zero word (every channel +1).
            const uint32_t* src = v ? rowp + static_cast<size_t>(wi) * G::D : g_zero_pixel;
#pragma unroll
            for (int d = 0; d < G::D; ++d)
                buf[cc * G::D + d] = src[d];
        }
    }
}

template <int CW, int S, int P, int UNIT, int UD, int KD>
__device__ __forceinline__ void wreg_compute_unit(const uint32_t (&buf)[UD], int (&acc)[P],
                                                  const uint32_t (&wreg)[KD])
{
    using G = WregGeom<CW, S, P>;
    static_assert(UD == G::UD && KD == G::KD, "buffer sizes");
    constexpr int i = UNIT / G::UPR;
    constexpr int c0 = (UNIT % G::UPR) * G::UC;
#pragma unroll
    for (int cc = 0; cc < G::UC; ++cc) {
        const int c = c0 + cc;
        if (c < G::WIN) {
#pragma unroll
            for (int pp = 0; pp < P; ++pp) {
                const int j = c - pp * S;  // which kernel column this input column is for pixel pp
                if (j >= 0 && j < 3) {
                    xor_popc_acc<G::D>(acc[pp], &buf[cc * G::D], &wreg[(i * 3 + j) * G::D]);
                }
            }
        }
    }
}

template <int CW, int S, int P>
__global__ __launch_bounds__(256) void bconv3x3_wreg_kernel(
    const uint32_t* __restrict__ a, const uint32_t* __restrict__ w, int32_t* __restrict__ y,
    int H, int W, int Cout, int Ho, int Wo, int pad, int K, int chunks, int groups, int ranges,
    int base_tasks, int rem_tasks)
{
    using G = WregGeom<CW, S, P>;

    const int lane = threadIdx.x & 63;
    const int gw = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int cg = gw % groups;  // which 64 output channels
    const int r = gw / groups;   // which range of tasks
    if (r >= ranges)
        return;  // the grid is rounded up to whole workgroups
    // balanced contiguous partition: the first rem_tasks ranges hold one task more
    int t = r * base_tasks + (r < rem_tasks ? r : rem_tasks);
    const int t_end = t + base_tasks + (r < rem_tasks ? 1 : 0);
    if (t >= t_end)
        return;

    const int cout = cg * 64 + lane;
    const bool cvalid = cout < Cout;
    const int coutc = cvalid ? cout : Cout - 1;

    uint32_t wreg[G::KD];
    {
        const uint2* wp = reinterpret_cast<const uint2*>(w + static_cast<size_t>(coutc) * G::KD);
#pragma unroll
        for (int q = 0; q < G::KD / 2; ++q) {
            const uint2 u = wp[q];
            wreg[2 * q] = u.x;
            wreg[2 * q + 1] = u.y;
        }
    }

    TaskPos tp;
    {
        const int row = t / chunks;
        tp.chunk = t - row * chunks;
        tp.n = row / Ho;
        tp.ho = row - tp.n * Ho;
    }

    uint32_t buf0[G::UD], buf1[G::UD];
    wreg_load_unit<CW, S, P, 0>(buf0, a, tp, H, W, pad);

    for (; t < t_end; ++t) {
        TaskPos next = tp;
        if (++next.chunk == chunks) {
            next.chunk = 0;
            if (++next.ho == Ho) {
                next.ho = 0;
                ++next.n;
            }
        }

        int acc[P];
#pragma unroll
        for (int pp = 0; pp < P; ++pp)
            acc[pp] = 0;

        // Software pipeline: while unit u is consumed by the VALU, unit u+1 is in flight.
        static_for<0, G::U>([&](auto uc) {
            constexpr int u = decltype(uc)::value;
            wait_scalar_loads();
            schedule_fence();
            if constexpr (u + 1 < G::U) {
                if constexpr (u % 2 == 0)
                    wreg_load_unit<CW, S, P, u + 1>(buf1, a, tp, H, W, pad);
                else
                    wreg_load_unit<CW, S, P, u + 1>(buf0, a, tp, H, W, pad);
            } else if constexpr (G::U % 2 == 0) {
                if (t + 1 < t_end)  // first unit of the next task, into the buffer it expects
                    wreg_load_unit<CW, S, P, 0>(buf0, a, next, H, W, pad);
            }
            schedule_fence();
            if constexpr (u % 2 == 0)
                wreg_compute_unit<CW, S, P, u>(buf0, acc, wreg);
            else
                wreg_compute_unit<CW, S, P, u>(buf1, acc, wreg);
            schedule_fence();
        });

        const int wo0 = tp.chunk * P;
        int32_t* yrow = y + ((static_cast<size_t>(tp.n) * Ho + tp.ho) * Wo + wo0) * Cout;
#pragma unroll
        for (int pp = 0; pp < P; ++pp) {
            if (wo0 + pp < Wo && cvalid)
                yrow[static_cast<unsigned>(pp * Cout + cout)] = K - 2 * acc[pp];
        }

        tp = next;
        if constexpr (G::U % 2 != 0) {
            if (t + 1 < t_end)
                wreg_load_unit<CW, S, P, 0>(buf0, a, tp, H, W, pad);
        }
    }
}

template <int CW, int S, int P>
hipError_t launch_wreg_inst(const uint32_t* a, const uint32_t* w, int32_t* y, const ConvShape& s,
                            hipStream_t stream)
{
    auto kernel = bconv3x3_wreg_kernel<CW, S, P>;
    static const int blocks_per_cu = resident_blocks_per_cu(kernel);
    const int chunks = (s.Wo + P - 1) / P;
    const int64_t n_tasks64 = static_cast<int64_t>(s.N) * s.Ho * chunks;
    if (n_tasks64 > 0x3fffffff)
        return hipErrorNotSupported;
    const int n_tasks = static_cast<int>(n_tasks64);
    const int groups = (s.Cout + 63) / 64;
    // Resident wavefront slots, split between channel groups; every range gets the same number
    // of tasks (+-1), so all wavefronts finish together in a single resident round.
    const int64_t slots = static_cast<int64_t>(blocks_per_cu) * device_cu_count() * 4;
    int ranges = static_cast<int>(slots / groups);
    if (ranges < 1)
        ranges = 1;
    if (ranges > n_tasks)
        ranges = n_tasks;
    const int base_tasks = n_tasks / ranges;
    const int rem_tasks = n_tasks % ranges;
    const int64_t waves = static_cast<int64_t>(ranges) * groups;
    const dim3 grid(static_cast<unsigned>((waves + 3) / 4)), block(256);
    hipLaunchKernelGGL(kernel, grid, block, 0, stream, a, w, y, s.H, s.W, s.Cout, s.Ho, s.Wo, s.pad,
                       s.K, chunks, groups, ranges, base_tasks, rem_tasks);
    return hipGetLastError();
}

template <int CW, int S>
hipError_t launch_wreg_p(const uint32_t* a, const uint32_t* w, int32_t* y, const ConvShape& s,
                         hipStream_t stream)
{
    // Pick the chunk width that wastes the fewest output columns (ties: the wider one).
    const int waste8 = (s.Wo + 7) / 8 * 8 - s.Wo;
    const int waste7 = (s.Wo + 6) / 7 * 7 - s.Wo;
    int p = (waste7 < waste8) ? 7 : 8;
    const int forced = option(DABNN_OPT_WREG_PIXELS);  // 0: as above; 7 or 8 forces the chunk width
    if (forced == 7 || forced == 8)
        p = forced;
    if (p == 7)
        return launch_wreg_inst<CW, S, 7>(a, w, y, s, stream);
    return launch_wreg_inst<CW, S, 8>(a, w, y, s, stream);
}

template <int CW>
hipError_t launch_wreg_s(const uint32_t* a, const uint32_t* w, int32_t* y, const ConvShape& s,
                         hipStream_t stream)
{
    if (s.stride == 1)
        return launch_wreg_p<CW, 1>(a, w, y, s, stream);
    return launch_wreg_p<CW, 2>(a, w, y, s, stream);
}

}  // namespace

hipError_t launch_bconv_reference(const uint64_t* a, const uint64_t* w, int32_t* y,
                                  const ConvShape& s, hipStream_t stream)
{
    const int64_t total = static_cast<int64_t>(s.N) * s.Ho * s.Wo * s.Cout;
    const int64_t blocks = (total + 255) / 256;
    bconv_reference_kernel<<<dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream>>>(a, w, y, s,
                                                                                         total);
    return hipGetLastError();
}

hipError_t launch_bconv_bnsign_reference(const uint64_t* a, const uint64_t* w, const int32_t* thr,
                                         const uint64_t* flip, uint64_t* out, const ConvShape& s,
                                         hipStream_t stream)
{
    const int64_t total = static_cast<int64_t>(s.N) * s.Ho * s.Wo * ((s.Cout + 63) / 64);
    const int64_t blocks = (total + 255) / 256;
    bconv_bnsign_reference_kernel<<<dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream>>>(
        a, w, thr, flip, out, s, total);
    return hipGetLastError();
}

bool bconv_wreg_supports(const ConvShape& s)
{
    return s.kh == 3 && s.kw == 3 && (s.stride == 1 || s.stride == 2) &&
           (s.Cw == 1 || s.Cw == 2 || s.Cw == 4 || s.Cw == 8);
}

hipError_t launch_bconv_wreg(const uint64_t* a, const uint64_t* w, int32_t* y, const ConvShape& s,
                             hipStream_t stream)
{
    if (!bconv_wreg_supports(s))
        return hipErrorNotSupported;
    const uint32_t* a32 = reinterpret_cast<const uint32_t*>(a);
    const uint32_t* w32 = reinterpret_cast<const uint32_t*>(w);
    switch (s.Cw) {
        case 1: return launch_wreg_s<1>(a32, w32, y, s, stream);
        case 2: return launch_wreg_s<2>(a32, w32, y, s, stream);
        case 4: return launch_wreg_s<4>(a32, w32, y, s, stream);
        default: return launch_wreg_s<8>(a32, w32, y, s, stream);
    }
}

}  // namespace dabnn

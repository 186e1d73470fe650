// Binary direct convolution (Sec. 2.1.2, Eq. 6-7), "activation-stationary" kernel family.
//
// Lane l of a wavefront owns one output pixel and keeps the 3x3xCin window under it (18*Cw
// dwords, out-of-image taps as zero words) in VGPRs -- the paper's idea of holding the window
// in registers while it is reused (Fig. 3), here reused across OUTPUT CHANNELS instead of across
// neighbouring pixels.  The wavefront then walks over output channels: the packed filter words
// are the same for all 64 lanes, so they are fetched with scalar loads and used as the SGPR
// operand of v_xor_b32, followed by v_bcnt_u32_b32 which accumulates the popcount (Eq. 6).  Four
// output channels are computed together (four independent accumulation chains) and written as
// one 16-byte store per lane.  All border handling happens once per window load; the hot loop
// contains no address arithmetic, no masks and no LDS.
//
// This family suits layers with few words per pixel (small windows, small filters that stay in
// the scalar cache); the filter-stationary family in bconv.hip suits the opposite case.
#include "kernel_util.h"
#include "launch.h"

namespace dabnn {
namespace {

// acc[q] += sum_{d<3} popcount(w[q][d] ^ a[d]) for four output channels q.  w sits in SGPRs
// (written by scalar loads only: a VALU-written SGPR would need wait states the compiler cannot
// see inside the assembly), a in VGPRs.  Four independent chains hide the VALU latency.
__device__ __forceinline__ void xor_popc_4x3(int* acc, const uint32_t* a, const uint32_t* w0,
                                             const uint32_t* w1, const uint32_t* w2,
                                             const uint32_t* w3)
{
    uint32_t t0, t1, t2, t3;
    asm("v_xor_b32 %4, %11, %8\n\t"
        "v_xor_b32 %5, %14, %8\n\t"
        "v_xor_b32 %6, %17, %8\n\t"
        "v_xor_b32 %7, %20, %8\n\t"
        "v_bcnt_u32_b32 %0, %4, %0\n\t"
        "v_bcnt_u32_b32 %1, %5, %1\n\t"
        "v_bcnt_u32_b32 %2, %6, %2\n\t"
        "v_bcnt_u32_b32 %3, %7, %3\n\t"
        "v_xor_b32 %4, %12, %9\n\t"
        "v_xor_b32 %5, %15, %9\n\t"
        "v_xor_b32 %6, %18, %9\n\t"
        "v_xor_b32 %7, %21, %9\n\t"
        "v_bcnt_u32_b32 %0, %4, %0\n\t"
        "v_bcnt_u32_b32 %1, %5, %1\n\t"
        "v_bcnt_u32_b32 %2, %6, %2\n\t"
        "v_bcnt_u32_b32 %3, %7, %3\n\t"
        "v_xor_b32 %4, %13, %10\n\t"
        "v_xor_b32 %5, %16, %10\n\t"
        "v_xor_b32 %6, %19, %10\n\t"
        "v_xor_b32 %7, %22, %10\n\t"
        "v_bcnt_u32_b32 %0, %4, %0\n\t"
        "v_bcnt_u32_b32 %1, %5, %1\n\t"
        "v_bcnt_u32_b32 %2, %6, %2\n\t"
        "v_bcnt_u32_b32 %3, %7, %3"
        : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "=&v"(t0), "=&v"(t1), "=&v"(t2),
          "=&v"(t3)
        : "v"(a[0]), "v"(a[1]), "v"(a[2]), "s"(w0[0]), "s"(w0[1]), "s"(w0[2]), "s"(w1[0]),
          "s"(w1[1]), "s"(w1[2]), "s"(w2[0]), "s"(w2[1]), "s"(w2[2]), "s"(w3[0]), "s"(w3[1]),
          "s"(w3[2]));
}

// The same for two output channels and six dwords: operands %0-%1 accumulators, %2-%5
// temporaries, %6-%11 activation dwords, %12-%17 / %18-%23 the two filters' dwords.
#define DABNN_P2(A0, A1, W0A, W1A, W0B, W1B)                \
    "v_xor_b32 %2, %" #W0A ", %" #A0 "\n\t"                 \
    "v_xor_b32 %3, %" #W1A ", %" #A0 "\n\t"                 \
    "v_xor_b32 %4, %" #W0B ", %" #A1 "\n\t"                 \
    "v_xor_b32 %5, %" #W1B ", %" #A1 "\n\t"                 \
    "v_bcnt_u32_b32 %0, %2, %0\n\t"                         \
    "v_bcnt_u32_b32 %1, %3, %1\n\t"                         \
    "v_bcnt_u32_b32 %0, %4, %0\n\t"                         \
    "v_bcnt_u32_b32 %1, %5, %1\n\t"
__device__ __forceinline__ void xor_popc_2x6(int* acc, const uint32_t* a, const uint32_t* w0,
                                             const uint32_t* w1)
{
    uint32_t t0, t1, t2, t3;
    asm(DABNN_P2(6, 7, 12, 18, 13, 19) DABNN_P2(8, 9, 14, 20, 15, 21) DABNN_P2(10, 11, 16, 22, 17, 23)
        : "+v"(acc[0]), "+v"(acc[1]), "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3)
        : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "s"(w0[0]), "s"(w0[1]),
          "s"(w0[2]), "s"(w0[3]), "s"(w0[4]), "s"(w0[5]), "s"(w1[0]), "s"(w1[1]), "s"(w1[2]),
          "s"(w1[3]), "s"(w1[4]), "s"(w1[5]));
}
#undef DABNN_P2

// Geometry.  A group = CG output channels (the unit of work distribution and of the 16-byte
// stores); it is consumed in software-pipeline units of NQ channels x DC dwords of K.
//   V = 0: 4 channels x 6 dwords     V = 1: 2 channels x 18 dwords     V = 2: 4 channels x 9 dwords
template <int CW, int V>
struct AregGeom {
    static constexpr int D = 2 * CW;
    static constexpr int KD = 18 * CW;
    static constexpr int NQ = (V == 1) ? 2 : 4;
    static constexpr int DC = (V == 0) ? 6 : (V == 1) ? 18 : 9;
    static constexpr int CG = (V == 0 && CW == 1) ? 8 : 4;
    static constexpr int CHUNKS = KD / DC;               // units per NQ channels
    static constexpr int UNITS = (CG / NQ) * CHUNKS;     // units per group (always even)
    static constexpr int SB = NQ * DC;                   // SGPRs per unit buffer
};

// Scalar loads of unit UNIT of the group starting at output channel cout0.
template <int CW, int V, int UNIT, int SB>
__device__ __forceinline__ void areg_load_unit(uint32_t (&sb)[SB], const uint32_t* __restrict__ w,
                                               int cout0)
{
    using G = AregGeom<CW, V>;
    constexpr int sub = UNIT / G::CHUNKS;
    constexpr int chunk = UNIT % G::CHUNKS;
    const uint32_t* src = w + static_cast<size_t>(cout0 + G::NQ * sub) * G::KD + chunk * G::DC;
#pragma unroll
    for (int q = 0; q < G::NQ; ++q) {
#pragma unroll
        for (int d = 0; d < G::DC; ++d)
            sb[q * G::DC + d] = src[q * G::KD + d];
    }
}

template <int CW, int V, int UNIT, int SB, int KD, int CG>
__device__ __forceinline__ void areg_compute_unit(const uint32_t (&sb)[SB], int (&acc)[CG],
                                                  const uint32_t (&areg)[KD])
{
    using G = AregGeom<CW, V>;
    constexpr int sub = UNIT / G::CHUNKS;
    constexpr int chunk = UNIT % G::CHUNKS;
    int* qa = &acc[G::NQ * sub];
    const uint32_t* av = &areg[chunk * G::DC];
    if constexpr (G::NQ == 4) {
#pragma unroll
        for (int h = 0; h < G::DC; h += 3)
            xor_popc_4x3(qa, av + h, &sb[0 * G::DC + h], &sb[1 * G::DC + h], &sb[2 * G::DC + h],
                         &sb[3 * G::DC + h]);
    } else {
#pragma unroll
        for (int h = 0; h < G::DC; h += 6)
            xor_popc_2x6(qa, av + h, &sb[0 * G::DC + h], &sb[1 * G::DC + h]);
    }
}

template <int CW, int S, int V>
__global__ __launch_bounds__(256) void bconv3x3_areg_kernel(
    const uint32_t* __restrict__ a, const uint32_t* __restrict__ w, int32_t* __restrict__ y,
    int H, int W, int Cout, int Ho, int Wo, int pad, int K, int total_pix, int groups_per_tile,
    int n_ranges, int base_groups, int rem_groups, int dbg)
{
    using G = AregGeom<CW, V>;
    const int lane = threadIdx.x & 63;
    const int gw = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (gw >= n_ranges)
        return;  // the grid is rounded up to whole workgroups
    // balanced contiguous partition of (tile, channel group) pairs, channel group fastest
    int g = gw * base_groups + (gw < rem_groups ? gw : rem_groups);
    const int g_end = g + base_groups + (gw < rem_groups ? 1 : 0);
    if (g >= g_end)
        return;
    int tile = g / groups_per_tile;
    int cgi = g - tile * groups_per_tile;

    uint32_t areg[G::KD];
    bool pvalid = false;
    uint32_t ybase = 0;
    // The 3x3xCw window under this lane's output pixel; taps outside the image become zero
    // words (every channel +1).
    auto load_window = [&](int t) {
        const int p = t * 64 + lane;
        pvalid = p < total_pix;
        const int pc = pvalid ? p : total_pix - 1;
        const int n = pc / (Ho * Wo);
        const int r = pc - n * (Ho * Wo);
        const int ho = r / Wo;
        const int wo = r - ho * Wo;
        ybase = static_cast<uint32_t>(pc) * static_cast<uint32_t>(Cout);
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const int hi = ho * S - pad + i;
            const bool rv = static_cast<unsigned>(hi) < static_cast<unsigned>(H);
            const int hic = rv ? hi : 0;
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const int wi = wo * S - pad + j;
                const bool v = rv && static_cast<unsigned>(wi) < static_cast<unsigned>(W);
                const int wic = v ? wi : 0;
                const uint32_t keep = v ? 0xffffffffu : 0u;
                const uint32_t* src =
                    a + (static_cast<size_t>(n * H + hic) * W + wic) * G::D;
                if constexpr (G::D == 2) {
                    const uint2 u = *reinterpret_cast<const uint2*>(src);
                    areg[(i * 3 + j) * 2 + 0] = u.x & keep;
                    areg[(i * 3 + j) * 2 + 1] = u.y & keep;
                } else {
#pragma unroll
                    for (int d = 0; d < G::D; d += 4) {
                        const uint4 u = *reinterpret_cast<const uint4*>(src + d);
                        areg[(i * 3 + j) * G::D + d + 0] = u.x & keep;
                        areg[(i * 3 + j) * G::D + d + 1] = u.y & keep;
                        areg[(i * 3 + j) * G::D + d + 2] = u.z & keep;
                        areg[(i * 3 + j) * G::D + d + 3] = u.w & keep;
                    }
                }
            }
        }
    };
    load_window(tile);

    uint32_t sb0[G::SB], sb1[G::SB];
    areg_load_unit<CW, V, 0>(sb0, w, cgi * G::CG);

    for (; g < g_end; ++g) {
        int ncgi = cgi + 1, ntile = tile;
        if (ncgi == groups_per_tile) {
            ncgi = 0;
            ++ntile;
        }

        int acc[G::CG];
#pragma unroll
        for (int q = 0; q < G::CG; ++q)
            acc[q] = 0;

        // Software pipeline: while unit u feeds the VALU, unit u+1 is in flight.
        static_for<0, G::UNITS>([&](auto uc) {
            constexpr int u = decltype(uc)::value;
            wait_scalar_loads();
            schedule_fence();
            if (dbg & 2) {
            } else if constexpr (u + 1 < G::UNITS) {
                if constexpr (u % 2 == 0)
                    areg_load_unit<CW, V, u + 1>(sb1, w, cgi * G::CG);
                else
                    areg_load_unit<CW, V, u + 1>(sb0, w, cgi * G::CG);
            } else {
                if (g + 1 < g_end)  // first unit of the next group (UNITS is even: buffer 0)
                    areg_load_unit<CW, V, 0>(sb0, w, ncgi * G::CG);
            }
            schedule_fence();
            if constexpr (u % 2 == 0)
                areg_compute_unit<CW, V, u>(sb0, acc, areg);
            else
                areg_compute_unit<CW, V, u>(sb1, acc, areg);
            schedule_fence();
        });

        if (pvalid && !((dbg & 1) && acc[0] != 12345)) {
            int32_t* dst = y + ybase + static_cast<uint32_t>(cgi * G::CG);
#pragma unroll
            for (int q = 0; q < G::CG; q += 4) {
                int4 o;
                o.x = __mul24(acc[q + 0], -2) + K;  // one v_mad_i32_i24; acc <= K < 2^23
                o.y = __mul24(acc[q + 1], -2) + K;
                o.z = __mul24(acc[q + 2], -2) + K;
                o.w = __mul24(acc[q + 3], -2) + K;
                *reinterpret_cast<int4*>(dst + q) = o;
            }
        }

        if (ntile != tile)
            load_window(ntile);
        tile = ntile;
        cgi = ncgi;
    }
}

template <int CW, int S, int V>
hipError_t launch_areg_inst(const uint32_t* a, const uint32_t* w, int32_t* y, const ConvShape& s,
                            hipStream_t stream)
{
    using G = AregGeom<CW, V>;
    static_assert(G::UNITS % 2 == 0 && G::KD % G::DC == 0 && G::CG % G::NQ == 0, "pipeline geometry");
    auto kernel = bconv3x3_areg_kernel<CW, S, V>;
    static const int blocks_per_cu = resident_blocks_per_cu(kernel);
    const int64_t total_pix = static_cast<int64_t>(s.N) * s.Ho * s.Wo;
    const int64_t tiles = (total_pix + 63) / 64;
    const int groups_per_tile = s.Cout / G::CG;
    const int64_t n_groups64 = tiles * groups_per_tile;
    if (n_groups64 > 0x3fffffff)
        return hipErrorNotSupported;
    const int n_groups = static_cast<int>(n_groups64);
    // Exactly the resident wavefront slots; every wavefront gets the same number of groups
    // (+-1), so the launch is one balanced round.
    const int oversub = env_int("DABNN_AREG_OVERSUB", 1);
    int64_t ranges = static_cast<int64_t>(blocks_per_cu) * device_cu_count() * 4 * oversub;
    if (ranges > n_groups)
        ranges = n_groups;
    const int n_ranges = static_cast<int>(ranges);
    const int base_groups = n_groups / n_ranges;
    const int rem_groups = n_groups % n_ranges;
    const dim3 grid(static_cast<unsigned>((n_ranges + 3) / 4)), block(256);
    hipLaunchKernelGGL(kernel, grid, block, 0, stream, a, w, y, s.H, s.W, s.Cout, s.Ho, s.Wo, s.pad,
                       s.K, static_cast<int>(total_pix), groups_per_tile, n_ranges, base_groups,
                       rem_groups, env_int("DABNN_DBG", 0));
    return hipGetLastError();
}

template <int CW>
hipError_t launch_areg_s(const uint32_t* a, const uint32_t* w, int32_t* y, const ConvShape& s,
                         hipStream_t stream)
{
    const int v = env_int("DABNN_AREG_V", 0);
    if (s.stride == 1) {
        if (v == 1) return launch_areg_inst<CW, 1, 1>(a, w, y, s, stream);
        if (v == 2) return launch_areg_inst<CW, 1, 2>(a, w, y, s, stream);
        return launch_areg_inst<CW, 1, 0>(a, w, y, s, stream);
    }
    if (v == 1) return launch_areg_inst<CW, 2, 1>(a, w, y, s, stream);
    if (v == 2) return launch_areg_inst<CW, 2, 2>(a, w, y, s, stream);
    return launch_areg_inst<CW, 2, 0>(a, w, y, s, stream);
}

}  // namespace

bool bconv_areg_supports(const ConvShape& s, const void* y)
{
    if (!(s.kh == 3 && s.kw == 3 && (s.stride == 1 || s.stride == 2)))
        return false;
    if (!(s.Cw == 1 || s.Cw == 2 || s.Cw == 4))
        return false;
    const int cg = (s.Cw == 1) ? 8 : 4;
    return s.Cout % cg == 0 && (reinterpret_cast<uintptr_t>(y) & 15) == 0;
}

hipError_t launch_bconv_areg(const uint64_t* a, const uint64_t* w, int32_t* y, const ConvShape& s,
                             hipStream_t stream)
{
    if (!bconv_areg_supports(s, y))
        return hipErrorNotSupported;
    const uint32_t* a32 = reinterpret_cast<const uint32_t*>(a);
    const uint32_t* w32 = reinterpret_cast<const uint32_t*>(w);
    switch (s.Cw) {
        case 1: return launch_areg_s<1>(a32, w32, y, s, stream);
        case 2: return launch_areg_s<2>(a32, w32, y, s, stream);
        default: return launch_areg_s<4>(a32, w32, y, s, stream);
    }
}

}  // namespace dabnn

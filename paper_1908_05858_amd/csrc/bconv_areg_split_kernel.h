// Binary direct convolution (Sec. 2.1.2, Eq. 6-7), activation-stationary kernels in which the
// FOUR wavefronts of a workgroup share one (64-pixel tile, 16-channel group).
//
// bconv_areg_kernel.h keeps a pixel's whole 3x3 window in one lane's registers, which stops at 8
// words per pixel.  Here wavefront v of a workgroup holds only words [v*CWC, (v+1)*CWC) of every
// tap (18*CWC dwords per lane) and reads the same words of every filter through scalar loads;
// the four partial popcount sums of an output meet in LDS, once per output (Eq. 7's single
// reduction), and wavefront v finishes and stores pixels 16v .. 16v+15 of the tile.  A launch
// covers 4*CWC words starting at any word of the pixel and may ADD to y instead of writing it, so
// a tensor of any word count is covered by a few launches in a row (the first computes
// K - 2*P1, each further one adds -2*Pi).  In the launch over the last 1 to 3 words of a pixel
// only that many wavefronts have words to read (PARTIAL); the others contribute zero sums and
// take their share of the reduction and the stores.
//
// The inner step is the one of bconv_areg_kernel.h: v_xor_b32 with the filter word as SGPR
// operand, v_bcnt_u32_b32 accumulating, four channels at a time, scalar loads software-pipelined
// in units of 4 channels x 6 dwords.  Filter strides are run-time values here, so a unit's loads
// are "base + scalar byte offset".
#pragma once
#include "bconv_areg_common.h"

#include <algorithm>

namespace dabnn {
namespace {

// The three tensors are kernel parameters of their own: only a __restrict__ pointer parameter lets
// the compiler read the filters through scalar loads.
//   a : first packed word this launch reads of pixel 0
//   w : first packed word this launch reads of filter 0, tap 0
//   y : [N][Ho][Wo][Cout]
struct SplitArgs {
    int H, W, Ho, Wo, pad, stride;
    uint32_t pix_bytes;                // bytes from one pixel to the next: 8 * (words per pixel)
    uint32_t hw, hw_mul, hw_shift;     // Ho*Wo and its division constants
    uint32_t wo_mul, wo_shift;         // division constants of Wo
    int Cout, k_term, total_pix;       // k_term: K in the launch that writes y, 0 in one that adds
    int accumulate;
    int filter_bytes, tap_bytes;       // strides of the filter tensor
    int groups_per_tile;               // Cout / 16
    int n_groups, base_groups, rem_groups;   // work split over the workgroups of the launch
    int n_active;                      // PARTIAL: wavefronts that have words to read
    const int32_t* thr;                // BITS: per-channel thresholds and flip bits of the fused
    const uint64_t* flip;              //       threshold epilogue (y is then the packed output)
};

template <int CWC>
struct SplitGeom {
    static constexpr int D = 2 * CWC;     // window dwords per tap held by one wavefront
    static constexpr int KD = 18 * CWC;   // window dwords held by one wavefront
    static constexpr int CG = 16;
    static constexpr int CHUNKS = KD / kDC;
    static constexpr int UNITS = (CG / 4) * CHUNKS;   // units per group (always even)
    static constexpr int SB = 4 * kDC;
};

// Scalar loads of unit UNIT of the group starting at output channel cout0: 4 channels x 6 dwords
// of this wavefront's words, as 8-byte loads at 32-bit byte offsets from `wq` (the launcher checks
// that the filter tensor stays below 4 GiB).  The offsets are made opaque per unit, so that each
// unit forms its few offsets where it uses them: shared between units, the compiler would keep
// some two hundred of them live and spill scalar registers.
// CWT > 0: the launch covers a tensor of exactly CWT words per pixel, so the filter strides are
// compile-time constants and every load is "row pointer + immediate offset" -- no scalar
// arithmetic per load (the run-time strides cost some 36 scalar instructions per unit, which at 8
// words per pixel kept the CU's scalar unit half busy).
template <int CWC, int UNIT, int CWT, int SB>
__device__ __forceinline__ void split_load_unit(uint32_t (&sb)[SB], const uint32_t* __restrict__ wq,
                                                int cout0, int fs, int ts)
{
    using G = SplitGeom<CWC>;
    constexpr int quad = UNIT / G::CHUNKS;
    constexpr int chunk = UNIT % G::CHUNKS;
    if constexpr (CWT > 0) {
        constexpr int FS = 72 * CWT, TS = 8 * CWT;   // bytes per filter, bytes per tap
        const char* rowp = reinterpret_cast<const char*>(wq) + static_cast<size_t>(cout0 + 4 * quad) * FS;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
#pragma unroll
            for (int d = 0; d < kDC; d += 2) {
                const int f = chunk * kDC + d;
                const uint2 u = *reinterpret_cast<const uint2*>(rowp + q * FS + (f / G::D) * TS + (f % G::D) * 4);
                sb[q * kDC + d] = u.x;
                sb[q * kDC + d + 1] = u.y;
            }
        }
        return;
    }
    uint32_t row = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(cout0 + 4 * quad) *
                                                  static_cast<uint32_t>(fs));   // (uniform)
    asm volatile("" : "+s"(row), "+s"(fs), "+s"(ts));   // (fs, ts: by-value copies of this call)
    const char* base = reinterpret_cast<const char*>(wq);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
        for (int d = 0; d < kDC; d += 2) {   // one 64-bit word (never split over two taps)
            const int f = chunk * kDC + d;   // position in the wavefront's window
            const uint32_t off = row + static_cast<uint32_t>(q * fs + (f / G::D) * ts + (f % G::D) * 4);
            const uint2 u = *reinterpret_cast<const uint2*>(base + off);
            sb[q * kDC + d] = u.x;
            sb[q * kDC + d + 1] = u.y;
        }
    }
}

template <int CWC, int UNIT, int SB, int KD>
__device__ __forceinline__ void split_compute_unit(const uint32_t (&sb)[SB], int (&acc)[16],
                                                   const uint32_t (&areg)[KD])
{
    using G = SplitGeom<CWC>;
    constexpr int quad = UNIT / G::CHUNKS;
    constexpr int chunk = UNIT % G::CHUNKS;
    // the quad's accumulators are born in its first block: no zero-initialisation needed
    xor_popc_4x3<chunk == 0>(&acc[4 * quad], &areg[chunk * kDC], &sb[0 * kDC], &sb[1 * kDC],
                             &sb[2 * kDC], &sb[3 * kDC]);
    xor_popc_4x3<false>(&acc[4 * quad], &areg[chunk * kDC + 3], &sb[0 * kDC + 3], &sb[1 * kDC + 3],
                        &sb[2 * kDC + 3], &sb[3 * kDC + 3]);
}

// BITS: the fused threshold epilogue of dabnn_bconv2d_bnsign for a launch that covers all words of
// a pixel.  Instead of y the kernel writes the next layer's packed activations, bit c of a pixel
// = (y < thr[c]) XOR flip bit c: after the reduction lane (P, j) holds channels 4j..4j+3 of pixel
// P, forms their four bits, the four lanes of a pixel OR theirs together (two DPP quad permutes)
// and one of them stores the group's 16 bits.
template <int CWC, bool PARTIAL, bool BITS = false, int CWT = 0>
__global__ __launch_bounds__(256) void bconv3x3_areg_split_kernel(
    const uint32_t* __restrict__ a, const uint32_t* __restrict__ w, int32_t* __restrict__ y,
    const SplitArgs p)
{
    using G = SplitGeom<CWC>;
    static_assert(G::UNITS % 2 == 0 && G::KD % kDC == 0, "pipeline geometry");
    constexpr int CG = G::CG;
    __shared__ int32_t partial_lds[4 * 64 * CG];   // the four wavefronts' partial sums of a tile

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool active = !PARTIAL || wave < p.n_active;
    // What only the window load and the epilogue need is read from the kernel-argument segment
    // where it is used (scalar loads), instead of occupying SGPRs through the main loop: the
    // struct is the fourth kernel parameter, behind three pointers.
    auto args = []() {
        uint64_t addr = reinterpret_cast<uint64_t>(__builtin_amdgcn_kernarg_segment_ptr()) + 3 * sizeof(void*);
        asm volatile("" : "+s"(addr));  // re-read at every use: do not keep the fields in SGPRs
        return reinterpret_cast<const SplitArgs __attribute__((address_space(4)))*>(addr);
    };
    const int groups_per_tile = p.groups_per_tile, filter_bytes = p.filter_bytes, tap_bytes = p.tap_bytes;

    // this workgroup's (tile, group) pairs [g, g_end), channel group fastest; every workgroup
    // gets the same number (+-1)
    const int b = blockIdx.x;
    int g = b * p.base_groups + (b < p.rem_groups ? b : p.rem_groups);
    const int g_end = g + p.base_groups + (b < p.rem_groups ? 1 : 0);
    if (g >= g_end)
        return;   // uniform over the workgroup

    uint32_t areg[G::KD];
    // The 3x3 window under this lane's output pixel (this wavefront's words of it); taps outside
    // the image become zero words (every channel +1).
    auto load_window = [&](int tile) {
        const auto* q = args();
        const int px = tile * 64 + lane;
        const int pc = px < q->total_pix ? px : q->total_pix - 1;
        const int n = static_cast<int>(fast_div(static_cast<uint32_t>(pc), q->hw_mul, q->hw_shift));
        const int r = pc - n * static_cast<int>(q->hw);
        const int ho = static_cast<int>(fast_div(static_cast<uint32_t>(r), q->wo_mul, q->wo_shift));
        const int wo = r - ho * q->Wo;
        // Taps are addressed as a uniform base plus a 32-bit byte offset (the launcher checks that
        // the tensor fits); invalid taps read offset 0 and are masked.
        const int hi0 = ho * q->stride - q->pad, wi0 = wo * q->stride - q->pad;
        const uint32_t off0 = static_cast<uint32_t>((n * q->H + hi0) * q->W + wi0) * q->pix_bytes;
        const char* base = reinterpret_cast<const char*>(a) + wave * (CWC * 8);
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const bool rv = static_cast<unsigned>(hi0 + i) < static_cast<unsigned>(q->H);
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const bool v = rv && static_cast<unsigned>(wi0 + j) < static_cast<unsigned>(q->W);
                const uint32_t keep = v ? 0xffffffffu : 0u;
                const uint32_t off = v ? off0 + static_cast<uint32_t>(i * q->W + j) * q->pix_bytes : 0u;
                const char* src = base + off;
#pragma unroll
                for (int d = 0; d < G::D; d += 2) {   // pixels are 8-byte aligned: 8-byte loads
                    const uint2 u = *reinterpret_cast<const uint2*>(src + d * 4);
                    areg[(i * 3 + j) * G::D + d + 0] = u.x & keep;
                    areg[(i * 3 + j) * G::D + d + 1] = u.y & keep;
                }
            }
        }
    };
    // this wavefront's words of every filter tap
    const uint32_t* const wq = w + wave * G::D;

    int tile = g / groups_per_tile;
    int cgi = g - tile * groups_per_tile;
    uint32_t sb0[G::SB], sb1[G::SB];
    if (active) {
        load_window(tile);
        split_load_unit<CWC, 0, CWT>(sb0, wq, cgi * CG, filter_bytes, tap_bytes);
    }

    for (; g < g_end; ++g) {
        int ncgi = cgi + 1, ntile = tile;
        if (ncgi == groups_per_tile) {
            ncgi = 0;
            ++ntile;
        }
        int acc[CG];
        if (PARTIAL && !active) {
#pragma unroll
            for (int q = 0; q < CG; ++q)
                acc[q] = 0;
        }
        // Software pipeline: while unit u feeds the VALU, unit u+1 is in flight.
        if (active)
            static_for<0, G::UNITS>([&](auto uc) {
                constexpr int u = decltype(uc)::value;
                wait_scalar_loads();
                schedule_fence();
                if constexpr (u + 1 < G::UNITS) {
                    if constexpr (u % 2 == 0)
                        split_load_unit<CWC, u + 1, CWT>(sb1, wq, cgi * CG, filter_bytes, tap_bytes);
                    else
                        split_load_unit<CWC, u + 1, CWT>(sb0, wq, cgi * CG, filter_bytes, tap_bytes);
                } else {
                    if (g + 1 < g_end)  // first unit of the next group (UNITS is even: buffer 0)
                        split_load_unit<CWC, 0, CWT>(sb0, wq, ncgi * CG, filter_bytes, tap_bytes);
                }
                schedule_fence();
                if constexpr (u % 2 == 0)
                    split_compute_unit<CWC, u>(sb0, acc, areg);
                else
                    split_compute_unit<CWC, u>(sb1, acc, areg);
                schedule_fence();
            });

        // ---- reduction over the four wavefronts, then the store of a quarter each -------------
        // Row P of a wavefront's LDS slice holds pixel P's 16 partial sums as four 16-byte quads;
        // quad j sits in column j ^ swz(P) (no bank conflicts on the row-wise writes nor on the
        // reads below).  Lane (P, j) of wavefront v = P / 16 then adds the four partial quads of
        // its pixel and holds channels 4j .. 4j+3 of it: four neighbouring lanes write the 64
        // contiguous bytes of one pixel.
        auto swz = [](int P) { return (P >> 1) & 3; };
        {
            int32_t* slice = partial_lds + wave * (64 * CG);
            const int sw = swz(lane);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                *reinterpret_cast<int4*>(slice + lane * CG + 4 * (j ^ sw)) =
                    make_int4(acc[4 * j + 0], acc[4 * j + 1], acc[4 * j + 2], acc[4 * j + 3]);
        }
        __syncthreads();
        const int P = 16 * wave + (lane >> 2), j = lane & 3;
        int4 d = make_int4(0, 0, 0, 0);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int4 pv =
                *reinterpret_cast<const int4*>(partial_lds + v * (64 * CG) + P * CG + 4 * (j ^ swz(P)));
            d.x += pv.x;
            d.y += pv.y;
            d.z += pv.z;
            d.w += pv.w;
        }
        const auto* q = args();
        const int k_term = q->k_term;
        int4 o;
        o.x = finish_output(d.x, k_term);
        o.y = finish_output(d.y, k_term);
        o.z = finish_output(d.z, k_term);
        o.w = finish_output(d.w, k_term);
        if constexpr (BITS) {
            const int4 t = *reinterpret_cast<const int4*>(q->thr + cgi * CG + 4 * j);
            uint32_t nib = (o.x < t.x ? 1u : 0u) | (o.y < t.y ? 2u : 0u) | (o.z < t.z ? 4u : 0u) |
                           (o.w < t.w ? 8u : 0u);
            nib <<= 4 * j;
            // OR over the four lanes of the pixel (lanes 4q..4q+3): xor-1 then xor-2 partners
            nib |= static_cast<uint32_t>(__builtin_amdgcn_mov_dpp(static_cast<int>(nib), 0xB1, 0xF, 0xF, true));
            nib |= static_cast<uint32_t>(__builtin_amdgcn_mov_dpp(static_cast<int>(nib), 0x4E, 0xF, 0xF, true));
            const uint32_t fl16 = static_cast<uint32_t>(q->flip[cgi >> 2] >> (16 * (cgi & 3))) & 0xffffu;
            if (tile * 64 + P < q->total_pix && j == 0)
                reinterpret_cast<uint16_t*>(y)[static_cast<size_t>(tile * 64 + P) * (q->Cout >> 4) + cgi] =
                    static_cast<uint16_t>(nib ^ fl16);
        } else if (tile * 64 + P < q->total_pix) {
            int32_t* dst = y + static_cast<size_t>(tile * 64 + P) * q->Cout + cgi * CG + 4 * j;
            if (q->accumulate) {
                const int4 old = *reinterpret_cast<const int4*>(dst);
                o.x += old.x;
                o.y += old.y;
                o.z += old.z;
                o.w += old.w;
            }
            store_out4<true>(dst, o);
        }
        __syncthreads();   // the slices are free for the next group's partial sums

        if (ntile != tile && active && g + 1 < g_end)
            load_window(ntile);
        tile = ntile;
        cgi = ncgi;
    }
}

// One launch over words [word0, word0 + 4*CWC) (PARTIAL: [word0, word0 + active_waves)) of the
// cw_total words of every pixel and filter tap.
struct SplitLaunch {
    const uint32_t* a;   // packed activations, pixel 0 word 0
    const uint32_t* w;   // packed filters, filter 0 tap 0 word 0
    int32_t* y;
    int cw_total;
    int word0;
    bool first;          // writes y = K - 2*P; otherwise adds -2*P to y
    int active_waves;    // 4, or 1..3 with PARTIAL
    const int32_t* thr = nullptr;    // BITS: thresholds and flip bits; y is the packed output
    const uint64_t* flip = nullptr;
};

template <int CWC, bool PARTIAL, bool BITS = false, int CWT = 0>
hipError_t launch_split_inst(const SplitLaunch& L, const ConvShape& s, hipStream_t stream)
{
    auto kernel = bconv3x3_areg_split_kernel<CWC, PARTIAL, BITS, CWT>;
    static const int blocks_per_cu = resident_blocks_per_cu(kernel);
    const int64_t total_pix = static_cast<int64_t>(s.N) * s.Ho * s.Wo;
    const int64_t tiles = (total_pix + 63) / 64;
    const int groups_per_tile = s.Cout / 16;
    const int64_t n_groups64 = tiles * groups_per_tile;
    if (n_groups64 > 0x3fffffff)
        return hipErrorNotSupported;
    const int n_groups = static_cast<int>(n_groups64);
    // More (shorter) ranges than workgroups fit the chip, a whole number per CU; the hardware's
    // dispatcher hands them out as slots free up (see launch_areg_inst in bconv_areg_kernel.h).
    int64_t per_cu = std::max(7, blocks_per_cu + 3);
    if (option(DABNN_OPT_AREG_RANGES_PER_SIMD) > 0)
        per_cu = option(DABNN_OPT_AREG_RANGES_PER_SIMD);
    if (per_cu * device_cu_count() > n_groups)
        per_cu = std::max<int64_t>(n_groups / device_cu_count(), 1);
    int64_t blocks = per_cu * device_cu_count();
    const int forced_slots = option(DABNN_OPT_AREG_SLOTS);   // > 0: that many wavefronts
    if (forced_slots > 0)
        blocks = (forced_slots + 3) / 4;
    if (blocks > n_groups)
        blocks = n_groups;

    SplitArgs p{};
    p.H = s.H;
    p.W = s.W;
    p.Ho = s.Ho;
    p.Wo = s.Wo;
    p.pad = s.pad;
    p.stride = s.stride;
    p.pix_bytes = static_cast<uint32_t>(L.cw_total) * 8u;
    p.hw = static_cast<uint32_t>(s.Ho) * static_cast<uint32_t>(s.Wo);
    division_constants(p.hw, p.hw_mul, p.hw_shift);
    division_constants(static_cast<uint32_t>(s.Wo), p.wo_mul, p.wo_shift);
    p.Cout = s.Cout;
    p.k_term = L.first ? s.K : 0;
    p.total_pix = static_cast<int>(total_pix);
    p.accumulate = L.first ? 0 : 1;
    p.filter_bytes = 72 * L.cw_total;
    p.tap_bytes = 8 * L.cw_total;
    p.groups_per_tile = groups_per_tile;
    p.n_groups = n_groups;
    p.base_groups = n_groups / static_cast<int>(blocks);
    p.rem_groups = n_groups % static_cast<int>(blocks);
    p.n_active = L.active_waves;
    p.thr = L.thr;
    p.flip = L.flip;
    hipLaunchKernelGGL(kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream,
                       L.a + 2 * L.word0, L.w + 2 * L.word0, L.y, p);
    return hipGetLastError();
}

}  // namespace

// One translation unit per CWC instantiates its kernels and exports this entry point;
// bconv_areg.hip dispatches to them.
#define DABNN_DEFINE_SPLIT_ENTRY_POINT(CWC, ...)                                                   \
    hipError_t launch_split_cw##CWC(const uint32_t* a, const uint32_t* w, int32_t* y, int cw_total, \
                                    int word0, bool first, int active_waves, const ConvShape& s,   \
                                    hipStream_t stream)                                            \
    {                                                                                              \
        const SplitLaunch L{a, w, y, cw_total, word0, first, active_waves};                        \
        __VA_ARGS__                                                                                \
        return launch_split_inst<CWC, false>(L, s, stream);                                        \
    }

}  // namespace dabnn

// Binary direct convolution (Sec. 2.1.2, Eq. 6-7), "activation-stationary" kernel family.
//
// Lane l of a wavefront owns one output pixel and keeps the 3x3xCin window under it (18*Cw
// dwords, out-of-image taps as zero words) in VGPRs -- the paper's idea of holding the window
// in registers while it is reused (Fig. 3), here reused across OUTPUT CHANNELS instead of across
// neighbouring pixels.  The wavefront then walks over output channels: the packed filter words
// are the same for all 64 lanes, so they are fetched with scalar loads and used as the SGPR
// operand of v_xor_b32, followed by v_bcnt_u32_b32 which accumulates the popcount (Eq. 6).  Four
// output channels are computed together (four independent accumulation chains).  All border
// handling happens once per window load; the hot loop contains no address arithmetic, no masks
// and no LDS.
//
// Stores: a lane holds consecutive channels of ONE pixel, so a direct store writes 16 bytes per
// lane at a stride of Cout*4 bytes -- 64 partial cache lines per instruction, which saturates the
// L2 write path long before HBM.  When Cout is a multiple of 16 the kernel therefore finishes 16
// channels, transposes the 64 x 16 tile through a wavefront-private slice of LDS and stores it so
// that four neighbouring lanes write the 64 contiguous bytes of one pixel.
//
// One wavefront holds a pixel's whole window here, which fits the register file up to 8 words per
// pixel (144 window registers).  bconv_areg_split_kernel.h spreads the words of a pixel over the
// four wavefronts of a workgroup and covers any word count.
#pragma once
#include "bconv_areg_common.h"

#include <algorithm>

namespace dabnn {
namespace {

// Geometry.  A group = CG output channels of one 64-pixel tile: the unit of work distribution
// and of the output stores.  It is consumed as CG/4 quads of channels; a quad's K dimension
// (18*Cw dwords) goes through the scalar-load software pipeline in units of 4 channels x 6 dwords.
//   TR = 16 (transposed store through LDS): CG = 16.   TR = 0, direct 16-byte stores:
//   CG = 4, or 8 when Cw is odd (which keeps the unit count even).   TR = kBits: fused threshold + bit-pack output, CG = 16 (a quarter of
//   an output word).
constexpr int kBits = -1;
constexpr int kRes = -3;    // fused BN + shortcut epilogue: float z and its packed sign bits
constexpr int kRes32 = -4;  // the same with 32 channels per group (128-byte runs of r and z)
constexpr bool is_res(int tr) { return tr == kRes || tr == kRes32; }

// What the window load needs, and nothing else does: the second kernel parameter.  The window
// is loaded once per 64-pixel tile, so these are fetched from the kernel-argument segment at that
// point (scalar loads) instead of occupying a dozen SGPRs through the main loop.  Divisions by
// Ho*Wo and Wo use multiply-shift constants prepared on the host.
struct WindowArgs {
    const uint32_t* a;
    int H, W, Ho, Wo, pad;
    uint32_t hw, hw_mul, hw_shift;  // Ho*Wo and its division constants
    uint32_t wo_mul, wo_shift;      // division constants of Wo
};

// Extra operands of the kRes mode.  It is the FIRST kernel parameter, so it sits at offset 0 of
// the kernel-argument segment and the epilogue can fetch its fields from there with scalar loads
// when it needs them, instead of holding ten more SGPRs through the main loop.
struct ResArgs {
    const float* scale;   // [Cout]
    const float* shift;   // [Cout]
    const float* r;       // [N][Ho][Wo][Cout], not null
    float* x_out;         // [N][Ho][Wo][Cout]
    uint16_t* bits16;     // the packed output viewed as [N*Ho*Wo][Cout/16] half-words
};
constexpr int kTailTR = 16;  // the store mode whose uneven remainder is split into small pieces
template <int CW, int TR>
struct AregGeom {
    static constexpr int D = 2 * CW;
    static constexpr int KD = 18 * CW;
    static constexpr int CG =
        TR > 0 ? TR : (TR == kRes32 ? 32 : ((TR == kBits || TR == kRes) ? 16 : (CW % 2 ? 8 : 4)));
    static constexpr int CHUNKS = KD / kDC;            // units per quad
    static constexpr int UNITS = (CG / 4) * CHUNKS;    // units per group (always even)
    static constexpr int SB = 4 * kDC;                 // SGPRs per unit buffer
};

// Scalar loads of unit UNIT of the group starting at output channel cout0.
template <int CW, int TR, int UNIT, int SB>
__device__ __forceinline__ void areg_load_unit(uint32_t (&sb)[SB], const uint32_t* __restrict__ w,
                                               int cout0)
{
    using G = AregGeom<CW, TR>;
    constexpr int quad = UNIT / G::CHUNKS;
    constexpr int chunk = UNIT % G::CHUNKS;
    const uint32_t* src = w + static_cast<size_t>(cout0 + 4 * quad) * G::KD + chunk * kDC;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
        for (int d = 0; d < kDC; ++d)
            sb[q * kDC + d] = src[q * G::KD + d];
    }
}

template <int CW, int TR, int UNIT, int SB, int KD, int CG>
__device__ __forceinline__ void areg_compute_unit(const uint32_t (&sb)[SB], int (&acc)[CG],
                                                  const uint32_t (&areg)[KD])
{
    using G = AregGeom<CW, TR>;
    constexpr int quad = UNIT / G::CHUNKS;
    constexpr int chunk = UNIT % G::CHUNKS;
    // the quad's accumulators are born in its first block: no zero-initialisation needed
    xor_popc_4x3<chunk == 0>(&acc[4 * quad], &areg[chunk * kDC], &sb[0 * kDC], &sb[1 * kDC],
                             &sb[2 * kDC], &sb[3 * kDC]);
    xor_popc_4x3<false>(&acc[4 * quad], &areg[chunk * kDC + 3], &sb[0 * kDC + 3], &sb[1 * kDC + 3],
                        &sb[2 * kDC + 3], &sb[3 * kDC + 3]);
}

template <int CW, int S, int TR>
__global__ __launch_bounds__(256) void bconv3x3_areg_kernel(
    ResArgs /* read through the kernel-argument segment, see ResArgs */,
    WindowArgs /* likewise, at offset sizeof(ResArgs) */,
    const uint32_t* __restrict__ w, int32_t* __restrict__ y,
    int Cout, int K, int total_pix, int groups_per_tile,
    int n_ranges, int base_groups, int rem_groups, int tail_first, int tail_base, int tail_rem,
    const int32_t* __restrict__ thr, const uint2* __restrict__ flip)
{
    // 64 pixels x TR channels of int32 per wavefront, used only by the transposed store
    __shared__ int32_t tile_lds[TR > 0 ? 4 * 64 * TR : (is_res(TR) ? 4 * 64 * AregGeom<CW, TR>::CG : 4)];

    // The kernel-argument segment spans three cache lines, and the first window load reads the
    // first of them only after the launch geometry (in the other two) has arrived and been
    // used: request it now, so that a launch starts with one memory round trip, not two.
    {
        const uint64_t ka_addr = reinterpret_cast<uint64_t>(__builtin_amdgcn_kernarg_segment_ptr());
        const uint32_t first_line =
            *reinterpret_cast<const uint32_t __attribute__((address_space(4)))*>(ka_addr);
        asm volatile("" : : "s"(first_line));
    }
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int gw = blockIdx.x * 4 + wave;
    if (gw >= n_ranges)
        return;  // the grid is rounded up to whole workgroups

    uint32_t areg[18 * CW];
    bool pvalid = false;
    uint32_t ybase = 0;
    // The 3x3xCw window under this lane's output pixel; taps outside the image become zero
    // words (every channel +1).
    auto load_window = [&](int t) {
        // the window operands, fetched now from the kernel-argument segment
        uint64_t wa_addr = reinterpret_cast<uint64_t>(__builtin_amdgcn_kernarg_segment_ptr()) + sizeof(ResArgs);
        asm volatile("" : "+s"(wa_addr));  // re-read per tile: do not keep the fields in SGPRs
        const auto* wa = reinterpret_cast<const WindowArgs __attribute__((address_space(4)))*>(wa_addr);
        const uint32_t* a = wa->a;
        const int H = wa->H, W = wa->W, pad = wa->pad;
        const int Wo = wa->Wo;
        const int p = t * 64 + lane;
        pvalid = p < total_pix;
        const int pc = pvalid ? p : total_pix - 1;
        const int n = static_cast<int>(fast_div(static_cast<uint32_t>(pc), wa->hw_mul, wa->hw_shift));
        const int r = pc - n * static_cast<int>(wa->hw);
        const int ho = static_cast<int>(fast_div(static_cast<uint32_t>(r), wa->wo_mul, wa->wo_shift));
        const int wo = r - ho * Wo;
        ybase = static_cast<uint32_t>(pc) * static_cast<uint32_t>(Cout);
        // Pixel index of the window's top-left tap; taps are addressed as a uniform base plus a
        // 32-bit byte offset (the launcher checks that the tensor fits), invalid taps read
        // offset 0 and are masked.
        const int hi0 = ho * S - pad, wi0 = wo * S - pad;
        const int top_left = (n * H + hi0) * W + wi0;
        const char* base = reinterpret_cast<const char*>(a);
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const bool rv = static_cast<unsigned>(hi0 + i) < static_cast<unsigned>(H);
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const bool v = rv && static_cast<unsigned>(wi0 + j) < static_cast<unsigned>(W);
                const uint32_t keep = v ? 0xffffffffu : 0u;
                const uint32_t off =
                    v ? static_cast<uint32_t>(top_left + i * W + j) * ((2 * CW) * 4u) : 0u;
                const char* src = base + off;
                if constexpr ((2 * CW) % 4 != 0) {
                    // an odd number of words: pixels are 8-byte aligned only, 8-byte loads
#pragma unroll
                    for (int d = 0; d < (2 * CW); d += 2) {
                        const uint2 u = *reinterpret_cast<const uint2*>(src + d * 4);
                        areg[(i * 3 + j) * (2 * CW) + d + 0] = u.x & keep;
                        areg[(i * 3 + j) * (2 * CW) + d + 1] = u.y & keep;
                    }
                } else {
#pragma unroll
                    for (int d = 0; d < (2 * CW); d += 4) {
                        const uint4 u = *reinterpret_cast<const uint4*>(src + d * 4);
                        areg[(i * 3 + j) * (2 * CW) + d + 0] = u.x & keep;
                        areg[(i * 3 + j) * (2 * CW) + d + 1] = u.y & keep;
                        areg[(i * 3 + j) * (2 * CW) + d + 2] = u.z & keep;
                        areg[(i * 3 + j) * (2 * CW) + d + 3] = u.w & keep;
                    }
                }
            }
        }
    };
    // Processes the (tile, channel group) pairs [g, g_end), channel group fastest, in store mode
    // TRX (its group size decides what a "group" is).
    auto run_range = [&](auto mode, int g, const int g_end, const int groups_per_tile) {
    constexpr int TRX = decltype(mode)::value;
    using G = AregGeom<CW, TRX>;
    if (g >= g_end)
        return;
    const int g_begin = g;
    int tile = g / groups_per_tile;
    int cgi = g - tile * groups_per_tile;
    load_window(tile);

    uint32_t sb0[G::SB], sb1[G::SB];
    areg_load_unit<CW, TRX, 0>(sb0, w, cgi * G::CG);
    uint32_t bits32 = 0;  // fused bit-pack output under construction

    for (; g < g_end; ++g) {
        int ncgi = cgi + 1, ntile = tile;
        if (ncgi == groups_per_tile) {
            ncgi = 0;
            ++ntile;
        }

        int acc[G::CG];
        // The group's 16 thresholds, fetched with vector loads at the start of the group (every
        // lane reads the same 64 bytes) so that they neither occupy SGPRs nor disturb the
        // scalar-load pipeline; they are first used after the last unit.
        int thr_v[TRX == kBits ? 16 : 1];
        if constexpr (TRX == kBits) {
            uint32_t lane_off = 0;
            asm volatile("" : "+v"(lane_off));  // keeps the address per-lane: a vector load
            const int4* tp = reinterpret_cast<const int4*>(thr + cgi * 16 + lane_off);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int4 t = tp[q];
                thr_v[4 * q + 0] = t.x;
                thr_v[4 * q + 1] = t.y;
                thr_v[4 * q + 2] = t.z;
                thr_v[4 * q + 3] = t.w;
            }
        }

        // kRes: the shortcut values this lane will need in the epilogue (QPR lanes per pixel:
        // pixel PPI*k + lane/QPR, channels 4*(lane%QPR)..+3 of this group), requested now so that
        // they arrive during the group's arithmetic.
        constexpr int RQPR = is_res(TRX) ? G::CG / 4 : 1;
        float4 r_pre[RQPR];
        if constexpr (is_res(TRX)) {
            const ResArgs* ka = (const ResArgs*)__builtin_amdgcn_kernarg_segment_ptr();
            const float* rp = ka->r;
#pragma unroll
            for (int k = 0; k < RQPR; ++k) {
                const int P = (64 / RQPR) * k + lane / RQPR;
                r_pre[k] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (tile * 64 + P < total_pix)
                    r_pre[k] = *reinterpret_cast<const float4*>(
                        rp + static_cast<size_t>(tile * 64 + P) * Cout + cgi * G::CG + 4 * (lane % RQPR));
            }
        }

        // Software pipeline: while unit u feeds the VALU, unit u+1 is in flight.
        static_for<0, G::UNITS>([&](auto uc) {
            constexpr int u = decltype(uc)::value;
            wait_scalar_loads();
            schedule_fence();
            if constexpr (u + 1 < G::UNITS) {
                if constexpr (u % 2 == 0)
                    areg_load_unit<CW, TRX, u + 1>(sb1, w, cgi * G::CG);
                else
                    areg_load_unit<CW, TRX, u + 1>(sb0, w, cgi * G::CG);
            } else {
                if (g + 1 < g_end)  // first unit of the next group (UNITS is even: buffer 0)
                    areg_load_unit<CW, TRX, 0>(sb0, w, ncgi * G::CG);
            }
            schedule_fence();
            if constexpr (u % 2 == 0)
                areg_compute_unit<CW, TRX, u>(sb0, acc, areg);
            else
                areg_compute_unit<CW, TRX, u>(sb1, acc, areg);
            schedule_fence();
        });

        if constexpr (TRX == kBits) {
            // Fused threshold + bit-pack: y < thr  <=>  (K - thr) - 2d < 0.  The 16 channels are
            // shifted in in ascending order and bit-reversed into place afterwards.  An even
            // group whose odd partner belongs to this wavefront too is held back, and the pair
            // leaves as one 32-bit store; a group whose partner belongs to a neighbouring
            // wavefront leaves as a 16-bit store (distinct bytes of the word: no race).
            const bool odd = (cgi & 1) != 0;
            if (!odd)
                bits32 = 0;
#pragma unroll
            for (int q = 0; q < 16; ++q)
                shift_in(bits32, acc[q], K - thr_v[q]);
            const uint2 fl = flip[cgi >> 2];
            const uint32_t fl32 = (cgi & 2) ? fl.y : fl.x;
            const size_t half_index =
                static_cast<size_t>(tile * 64 + lane) * (groups_per_tile >> 1) + (cgi >> 1);
            const uint32_t rev = __builtin_bitreverse32(bits32);
            if (odd && g > g_begin) {
                if (pvalid)
                    reinterpret_cast<uint32_t*>(y)[half_index] = rev ^ fl32;
            } else if (odd || g + 1 >= g_end) {
                const uint32_t fl16 = odd ? (fl32 >> 16) : (fl32 & 0xffffu);
                if (pvalid)
                    reinterpret_cast<uint16_t*>(y)[2 * half_index + (odd ? 1 : 0)] =
                        static_cast<uint16_t>((rev >> 16) ^ fl16);
            }
        } else if constexpr (is_res(TRX)) {
            // Fused BN + shortcut epilogue.  The 64 x CG tile of y goes through the LDS transpose
            // of the transposed store modes (CG = 16 or 32); afterwards lane (P, j) holds channels
            // 4j..4j+3 of pixel P, takes the matching 16 bytes of the shortcut, forms
            //   z = ((scale * float(y)) + shift) + r      (separately rounded: no FMA in this file)
            // stores z, and contributes 4 sign bits; the four lanes of a 16-channel quarter OR
            // them together and one of them stores those 16 bits.
            constexpr int CGR = G::CG;
            constexpr int QPR = CGR / 4;   // lanes per pixel
            constexpr int PPI = 64 / QPR;  // pixels per pass
            auto swz = [](int P) { return (CGR == 16) ? ((P >> 1) & 3) : (P & 7); };
            int32_t* slice = tile_lds + wave * (64 * CGR);
            {
                const int sw = swz(lane);
#pragma unroll
                for (int j = 0; j < QPR; ++j) {
                    int4 o;
                    o.x = finish_output(acc[4 * j + 0], K);
                    o.y = finish_output(acc[4 * j + 1], K);
                    o.z = finish_output(acc[4 * j + 2], K);
                    o.w = finish_output(acc[4 * j + 3], K);
                    *reinterpret_cast<int4*>(slice + lane * CGR + 4 * (j ^ sw)) = o;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            // the extra operands, fetched now from the kernel-argument segment (offset 0)
            const ResArgs* ka = (const ResArgs*)__builtin_amdgcn_kernarg_segment_ptr();
            const float* scale = ka->scale;
            const float* shift = ka->shift;
            float* xo = ka->x_out;
            uint16_t* bits16 = ka->bits16;
            const int j = lane % QPR;
            const int c0 = cgi * CGR + 4 * j;
            const float4 sc = *reinterpret_cast<const float4*>(scale + c0);
            const float4 sh = *reinterpret_cast<const float4*>(shift + c0);
            const uint32_t row0 = static_cast<uint32_t>(tile) * 64u;
#pragma unroll
            for (int k = 0; k < QPR; ++k) {
                const int P = PPI * k + lane / QPR;
                const int4 o = *reinterpret_cast<const int4*>(slice + P * CGR + 4 * (j ^ swz(P)));
                const bool ok = static_cast<int>(row0) + P < total_pix;
                const size_t e = static_cast<size_t>(row0 + P) * Cout + c0;
                const float4 rr = r_pre[k];
                float4 z;
                z.x = __fadd_rn(__fmul_rn(sc.x, static_cast<float>(o.x)), sh.x);
                z.y = __fadd_rn(__fmul_rn(sc.y, static_cast<float>(o.y)), sh.y);
                z.z = __fadd_rn(__fmul_rn(sc.z, static_cast<float>(o.z)), sh.z);
                z.w = __fadd_rn(__fmul_rn(sc.w, static_cast<float>(o.w)), sh.w);
                z.x = __fadd_rn(z.x, rr.x);
                z.y = __fadd_rn(z.y, rr.y);
                z.z = __fadd_rn(z.z, rr.z);
                z.w = __fadd_rn(z.w, rr.w);
                if (ok) {
                    typedef float v4f __attribute__((ext_vector_type(4)));
                    v4f zv = {z.x, z.y, z.z, z.w};
                    __builtin_nontemporal_store(zv, reinterpret_cast<v4f*>(xo + e));
                }
                uint32_t nib = (__float_as_uint(z.x) >> 31) | ((__float_as_uint(z.y) >> 31) << 1) |
                               ((__float_as_uint(z.z) >> 31) << 2) | ((__float_as_uint(z.w) >> 31) << 3);
                nib <<= 4 * (j & 3);
                // OR over the four lanes of a quarter (lanes 4q..4q+3): xor-1 then xor-2 partners
                nib |= static_cast<uint32_t>(__builtin_amdgcn_mov_dpp(static_cast<int>(nib), 0xB1, 0xF, 0xF, true));
                nib |= static_cast<uint32_t>(__builtin_amdgcn_mov_dpp(static_cast<int>(nib), 0x4E, 0xF, 0xF, true));
                if (ok && (j & 3) == 0)
                    bits16[static_cast<size_t>(row0 + P) * (Cout >> 4) + cgi * (CGR / 16) + (j >> 2)] =
                        static_cast<uint16_t>(nib);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        } else if constexpr (TRX != 0) {
            // Row P of the wavefront's LDS slice holds pixel P's TRX channels as QPR 16-byte quads.
            // Quad j sits in column j ^ swz(P), which makes both the row-wise writes and the
            // transposed reads free of bank conflicts (a 64-byte row covers half the banks, so
            // two neighbouring rows share one swizzle; a 128-byte row covers all of them).
            constexpr int QPR = TRX / 4;            // quads per row
            constexpr int LPP = QPR;               // lanes per pixel in the transposed store
            constexpr int PPI = 64 / LPP;          // pixels per store instruction
            auto swz = [](int P) { return (TRX == 16) ? ((P >> 1) & 3) : (P & 7); };
            int32_t* slice = tile_lds + wave * (64 * TRX);
            {
                const int sw = swz(lane);
#pragma unroll
                for (int j = 0; j < QPR; ++j) {
                    int4 o;
                    o.x = finish_output(acc[4 * j + 0], K);
                    o.y = finish_output(acc[4 * j + 1], K);
                    o.z = finish_output(acc[4 * j + 2], K);
                    o.w = finish_output(acc[4 * j + 3], K);
                    *reinterpret_cast<int4*>(slice + lane * TRX + 4 * (j ^ sw)) = o;
                }
            }
            // LDS instructions of one wavefront execute in order; this only stops the compiler
            // from moving the reads above the writes.
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const int j = lane % LPP;
            // uniform base + per-lane 32-bit byte offset; LPP neighbouring lanes write the
            // 4*TRX contiguous bytes of one pixel
            char* dst = reinterpret_cast<char*>(y + static_cast<size_t>(tile) * 64 * Cout + cgi * G::CG);
            if (tile * 64 + 64 <= total_pix) {  // whole tile inside the tensor (uniform)
                int4 o[LPP];
#pragma unroll
                for (int k = 0; k < LPP; ++k) {
                    const int P = PPI * k + lane / LPP;
                    o[k] = *reinterpret_cast<const int4*>(slice + P * TRX + 4 * (j ^ swz(P)));
                }
#pragma unroll
                for (int k = 0; k < LPP; ++k) {
                    const int P = PPI * k + lane / LPP;
                    store_out4<true>(dst + (static_cast<uint32_t>(P) * Cout + 4 * j) * 4u, o[k]);
                }
            } else {
#pragma unroll
                for (int k = 0; k < LPP; ++k) {
                    const int P = PPI * k + lane / LPP;
                    const int4 o = *reinterpret_cast<const int4*>(slice + P * TRX + 4 * (j ^ swz(P)));
                    if (tile * 64 + P < total_pix)
                        store_out4<true>(dst + (static_cast<uint32_t>(P) * Cout + 4 * j) * 4u, o);
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        } else {
            if (pvalid) {
                int32_t* dst = y + ybase + static_cast<uint32_t>(cgi * G::CG);
#pragma unroll
                for (int q = 0; q < G::CG; q += 4) {
                    int4 o;
                    o.x = finish_output(acc[q + 0], K);
                    o.y = finish_output(acc[q + 1], K);
                    o.z = finish_output(acc[q + 2], K);
                    o.w = finish_output(acc[q + 3], K);
                    store_out4<false>(dst + q, o);
                }
            }
        }

        if (ntile != tile)
            load_window(ntile);
        tile = ntile;
        cgi = ncgi;
    }
    };

    // Every wavefront first takes the same number (+-1) of whole groups, a contiguous range.
    const int g0 = gw * base_groups + (gw < rem_groups ? gw : rem_groups);
    run_range(std::integral_constant<int, TR>{}, g0, g0 + base_groups + (gw < rem_groups ? 1 : 0),
              groups_per_tile);
    // The groups that do not divide evenly over the wavefronts are handed out in pieces of 4 (or
    // 8) channels through the direct-store path, so that no wavefront -- and no SIMD -- carries a
    // whole extra group.
    if constexpr (TR == kTailTR) {
        using GT = AregGeom<CW, 0>;
        const int t0 = tail_first + gw * tail_base + (gw < tail_rem ? gw : tail_rem);
        run_range(std::integral_constant<int, 0>{}, t0, t0 + tail_base + (gw < tail_rem ? 1 : 0),
                  Cout / GT::CG);
    }
}

template <int CW, int S, int TR>
hipError_t launch_areg_inst(const uint32_t* a, const uint32_t* w, int32_t* y, const ConvShape& s,
                            hipStream_t stream, const int32_t* thr = nullptr,
                            const uint2* flip = nullptr, const ResArgs& res = ResArgs{})
{
    using G = AregGeom<CW, TR>;
    static_assert(G::UNITS % 2 == 0 && G::KD % kDC == 0, "pipeline geometry");
    auto kernel = bconv3x3_areg_kernel<CW, S, TR>;
    static const int blocks_per_cu = resident_blocks_per_cu(kernel);
    const int64_t total_pix = static_cast<int64_t>(s.N) * s.Ho * s.Wo;
    const int64_t tiles = (total_pix + 63) / 64;
    const int groups_per_tile = s.Cout / G::CG;
    const int64_t n_groups64 = tiles * groups_per_tile;
    if (n_groups64 > 0x3fffffff)
        return hipErrorNotSupported;
    const int n_groups = static_cast<int>(n_groups64);
    // The work is cut into contiguous ranges of groups, one per wavefront of the launch, every
    // range the same length (+-1).  A SIMD serves its oldest wavefront first, so wavefronts with
    // equal ranges do not end together: with exactly as many ranges as wavefronts fit the chip,
    // a SIMD runs the second half of the launch with ever fewer wavefronts to pick from.  With
    // more (shorter) ranges than resident wavefronts the hardware's dispatcher hands the rest out
    // as slots free up, which keeps every SIMD full until shortly before the end.  Measured at
    // batch 256 (ranges per SIMD: time): 1 word per pixel 7: 63 us, 10: 56 us; 4 words 4: 56 us,
    // 7: 55 us; 8 words 2: 63 us, 7: 58 us, 12: 61 us.  A whole number of ranges per SIMD keeps
    // the SIMDs' shares equal.
    const int simds = device_cu_count() * 4;
    int64_t per_simd = std::max(7, blocks_per_cu + 3);
    // A launch with less than 20 groups per SIMD: 7 ranges per SIMD whatever fits at once.  Ten
    // ranges of one or two groups each make the SIMDs' shares uneven and every range pays its
    // window load (measured, 12 groups per SIMD at one word per pixel: 64x56x56x64->64 17.7 us
    // against 20.8, 128x56x56x64->128 stride 2 17.1 against 19.2; no difference from 24 up).
    if (n_groups < 20 * simds)
        per_simd = 7;
    if (option(DABNN_OPT_AREG_RANGES_PER_SIMD) > 0)
        per_simd = option(DABNN_OPT_AREG_RANGES_PER_SIMD);
    if (per_simd * simds > n_groups)
        per_simd = std::max<int64_t>(n_groups / simds, 1);
    int64_t ranges = per_simd * simds;
    const int forced_slots = option(DABNN_OPT_AREG_SLOTS);  // > 0: that many ranges
    if (forced_slots > 0)
        ranges = forced_slots;
    if (ranges > n_groups)
        ranges = n_groups;
    const int n_ranges = static_cast<int>(ranges);
    const int base_groups = n_groups / n_ranges;
    int rem_groups = n_groups % n_ranges;
    // A small remainder (few wavefronts with a whole group more, i.e. a few SIMDs that finish a
    // group late) is instead split into direct-store pieces of 4 (8) channels and spread over
    // all wavefronts.  Measured at batch 256: -3 % kernel time at 14x14x256->256 (remainder
    // 6 % of the wavefronts); a large remainder is cheaper as whole groups, because the pieces
    // use the slower direct store and each needs its own window.
    int tail_first = 0, tail_base = 0, tail_rem = 0;
    const int tail_mode = option(DABNN_OPT_AREG_TAIL);  // 0 by size, 1 never, 2 always
    if (TR == kTailTR && rem_groups > 0 && tail_mode != 1 &&
        (tail_mode == 2 || rem_groups * 4 <= n_ranges)) {
        constexpr int pieces = G::CG / AregGeom<CW, 0>::CG;
        const int n_tail = rem_groups * pieces;
        tail_first = base_groups * n_ranges * pieces;
        tail_base = n_tail / n_ranges;
        tail_rem = n_tail % n_ranges;
        rem_groups = 0;
    }
    const dim3 grid(static_cast<unsigned>((n_ranges + 3) / 4)), block(256);
    WindowArgs wa{a, s.H, s.W, s.Ho, s.Wo, s.pad, 0, 0, 0, 0, 0};
    wa.hw = static_cast<uint32_t>(s.Ho) * static_cast<uint32_t>(s.Wo);
    division_constants(wa.hw, wa.hw_mul, wa.hw_shift);
    division_constants(static_cast<uint32_t>(s.Wo), wa.wo_mul, wa.wo_shift);
    hipLaunchKernelGGL(kernel, grid, block, 0, stream, res, wa, w, y, s.Cout,
                       s.K, static_cast<int>(total_pix), groups_per_tile, n_ranges, base_groups,
                       rem_groups, tail_first, tail_base, tail_rem, thr, flip);
    return hipGetLastError();
}

template <int CW, int S>
hipError_t launch_areg_s(const uint32_t* a, const uint32_t* w, int32_t* y, const ConvShape& s,
                         hipStream_t stream)
{
    // 16 channels transposed through LDS (64-byte runs) where Cout allows it.  With 8 words per
    // pixel (K = 4608) the output rate is so low that the direct store, which needs no LDS and
    // fewer registers, wins.
    int tr = (CW != 8 && s.Cout % 16 == 0) ? 16 : 0;
    // A launch with only a few 16-channel groups per SIMD (a single image, a small batch) is
    // bound by latency: its length is a few groups' arithmetic on the busiest SIMD.  Direct-store
    // groups are a quarter (half, for an odd word count) of that and there are four times (twice)
    // as many wavefronts.  Measured by HIP-graph replay, direct against transposed: 14x14x256->256
    // at batch 1: 4.4 against 8.9 us, at batch 32: 11.8 against 16.3; 56x56x64->64 at batch 8: 6.1
    // against 7.3, at batch 12 (2.3 groups per SIMD): 7.3 against 6.7.
    if (tr == 16 && bconv_areg_small_launch(s))
        tr = 0;
    const int forced = option(DABNN_OPT_AREG_STORE);  // 0 as above, 1 direct, 16 transposed
    if (forced == 1)
        tr = 0;
    else if (forced == 16 && s.Cout % 16 == 0)
        tr = 16;
    if (tr == 16) return launch_areg_inst<CW, S, 16>(a, w, y, s, stream);
    return launch_areg_inst<CW, S, 0>(a, w, y, s, stream);
}

}  // namespace

// One translation unit per (word count, stride) instantiates that combination's kernels and
// exports these two entry points; bconv_areg.hip dispatches to them.
#define DABNN_DEFINE_AREG_ENTRY_POINTS(CW, S)                                                     \
    hipError_t launch_areg_cw##CW##_s##S(const uint32_t* a, const uint32_t* w, int32_t* y,         \
                                         const ConvShape& s, hipStream_t stream)                  \
    {                                                                                             \
        return launch_areg_s<CW, S>(a, w, y, s, stream);                                          \
    }                                                                                             \
    hipError_t launch_bits_cw##CW##_s##S(const uint32_t* a, const uint32_t* w, uint64_t* out,      \
                                         const ConvShape& s, hipStream_t stream,                  \
                                         const int32_t* thr, const uint2* flip)                   \
    {                                                                                             \
        return launch_areg_inst<CW, S, kBits>(a, w, reinterpret_cast<int32_t*>(out), s, stream,   \
                                              thr, flip);                                         \
    }                                                                                             \
    hipError_t launch_res_cw##CW##_s##S(const uint32_t* a, const uint32_t* w, const ConvShape& s,  \
                                        hipStream_t stream, const float* scale,                   \
                                        const float* shift, const float* r, float* x_out,         \
                                        uint64_t* bits)                                           \
    {                                                                                             \
        const ResArgs res{scale, shift, r, x_out, reinterpret_cast<uint16_t*>(bits)};             \
        /* one word per pixel: the epilogue's r and z traffic dominates and 128-byte runs pay */  \
        if (CW == 1 && option(DABNN_OPT_RES_CHANNELS) != 16)                                    \
            return launch_areg_inst<CW, S, kRes32>(a, w, nullptr, s, stream, nullptr, nullptr,    \
                                                   res);                                          \
        return launch_areg_inst<CW, S, kRes>(a, w, nullptr, s, stream, nullptr, nullptr, res);    \
    }

}  // namespace dabnn

// Device and host helpers shared by the activation-stationary convolution kernels
// (bconv_areg_kernel.h: one wavefront per channel group; bconv_areg_split_kernel.h: the four
// wavefronts of a workgroup share a group).
#pragma once
#include "kernel_util.h"
#include "launch.h"

namespace dabnn {
namespace {

// acc[q] += sum_{d<3} popcount(w[q][d] ^ a[d]) for four output channels q.  w sits in SGPRs
// (written by scalar loads only: a VALU-written SGPR would need wait states the compiler cannot
// see inside the assembly), a in VGPRs.  Four independent chains hide the VALU latency.
template <bool FIRST>
__device__ __forceinline__ void xor_popc_4x3(int* acc, const uint32_t* a, const uint32_t* w0,
                                             const uint32_t* w1, const uint32_t* w2,
                                             const uint32_t* w3)
{
    uint32_t t0, t1, t2, t3;
#define DABNN_TAIL                                                                      \
    "v_xor_b32 %4, %12, %9\n\t"                                                         \
    "v_xor_b32 %5, %15, %9\n\t"                                                         \
    "v_xor_b32 %6, %18, %9\n\t"                                                         \
    "v_xor_b32 %7, %21, %9\n\t"                                                         \
    "v_bcnt_u32_b32 %0, %4, %0\n\t"                                                     \
    "v_bcnt_u32_b32 %1, %5, %1\n\t"                                                     \
    "v_bcnt_u32_b32 %2, %6, %2\n\t"                                                     \
    "v_bcnt_u32_b32 %3, %7, %3\n\t"                                                     \
    "v_xor_b32 %4, %13, %10\n\t"                                                        \
    "v_xor_b32 %5, %16, %10\n\t"                                                        \
    "v_xor_b32 %6, %19, %10\n\t"                                                        \
    "v_xor_b32 %7, %22, %10\n\t"                                                        \
    "v_bcnt_u32_b32 %0, %4, %0\n\t"                                                     \
    "v_bcnt_u32_b32 %1, %5, %1\n\t"                                                     \
    "v_bcnt_u32_b32 %2, %6, %2\n\t"                                                     \
    "v_bcnt_u32_b32 %3, %7, %3"
#define DABNN_INPUTS                                                                          \
    "v"(a[0]), "v"(a[1]), "v"(a[2]), "s"(w0[0]), "s"(w0[1]), "s"(w0[2]), "s"(w1[0]), "s"(w1[1]), \
        "s"(w1[2]), "s"(w2[0]), "s"(w2[1]), "s"(w2[2]), "s"(w3[0]), "s"(w3[1]), "s"(w3[2])
    if constexpr (FIRST) {
        // the accumulators start here: the first popcounts add to the constant 0
        asm("v_xor_b32 %4, %11, %8\n\t"
            "v_xor_b32 %5, %14, %8\n\t"
            "v_xor_b32 %6, %17, %8\n\t"
            "v_xor_b32 %7, %20, %8\n\t"
            "v_bcnt_u32_b32 %0, %4, 0\n\t"
            "v_bcnt_u32_b32 %1, %5, 0\n\t"
            "v_bcnt_u32_b32 %2, %6, 0\n\t"
            "v_bcnt_u32_b32 %3, %7, 0\n\t" DABNN_TAIL
            : "=&v"(acc[0]), "=&v"(acc[1]), "=&v"(acc[2]), "=&v"(acc[3]), "=&v"(t0), "=&v"(t1),
              "=&v"(t2), "=&v"(t3)
            : DABNN_INPUTS);
    } else {
        asm("v_xor_b32 %4, %11, %8\n\t"
            "v_xor_b32 %5, %14, %8\n\t"
            "v_xor_b32 %6, %17, %8\n\t"
            "v_xor_b32 %7, %20, %8\n\t"
            "v_bcnt_u32_b32 %0, %4, %0\n\t"
            "v_bcnt_u32_b32 %1, %5, %1\n\t"
            "v_bcnt_u32_b32 %2, %6, %2\n\t"
            "v_bcnt_u32_b32 %3, %7, %3\n\t" DABNN_TAIL
            : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "=&v"(t0), "=&v"(t1),
              "=&v"(t2), "=&v"(t3)
            : DABNN_INPUTS);
    }
#undef DABNN_TAIL
#undef DABNN_INPUTS
}

// y = K - 2 * diff as one v_mad_i32_i24 (diff <= K < 2^23).  K is a kernel argument, so the SGPR
// it sits in is written by a scalar load.
__device__ __forceinline__ int finish_output(int diff, int K)
{
    int y;
    asm("v_mad_i32_i24 %0, %1, -2, %2" : "=v"(y) : "v"(diff), "s"(K));
    return y;
}

// Outputs are written once and never read by this kernel.  The transposed path stores whole
// 64- or 128-byte runs, so it stores non-temporally (streaming through L2); the direct path
// writes 16-byte pieces of a line at different times and leaves it to L2 to merge them.
typedef int v4i __attribute__((ext_vector_type(4)));
template <bool STREAM>
__device__ __forceinline__ void store_out4(void* dst, const int4& o)
{
    v4i v = {o.x, o.y, o.z, o.w};
    if constexpr (STREAM)
        __builtin_nontemporal_store(v, reinterpret_cast<v4i*>(dst));
    else
        *reinterpret_cast<v4i*>(dst) = v;
}

// Fused threshold: bits = (bits << 1) | (y < thr) for one output channel, with y = K - 2d (d the
// popcount sum) and kt = K - thr:  y < thr  <=>  kt - 2d < 0.  Plain VALU arithmetic: the sign bit
// of kt - 2d is shifted in with v_alignbit_b32, no lane mask ever goes through an SGPR pair.
__device__ __forceinline__ void shift_in(uint32_t& bits, int d, int kt)
{
    const int t = kt - 2 * d;  // |kt|, 2d < 2^31: no overflow
    bits = __builtin_amdgcn_alignbit(bits, static_cast<uint32_t>(t), 31);
}

constexpr int kDC = 6;   // dwords per channel in one unit of the scalar-load pipeline

}  // namespace
}  // namespace dabnn

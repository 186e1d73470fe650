// Small device and host helpers shared by the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/dabnn.h"

#include <type_traits>

namespace dabnn {

// Compile-time loop: f(std::integral_constant<int, I>{}) for I in [I0, N).
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// Wait until every scalar load issued so far has landed (lgkmcnt = 0, other counters untouched).
__device__ __forceinline__ void wait_scalar_loads()
{
    __builtin_amdgcn_s_waitcnt(0xC07F);
}

// Nothing may be moved across this point by the instruction scheduler.
__device__ __forceinline__ void schedule_fence()
{
    __builtin_amdgcn_sched_barrier(0);
}

// floor(n / d) for any 32-bit n, with mul = floor(2^32 * (2^L - d) / d) + 1 and shift = L - 1,
// L = ceil(log2 d) (d = 1: mul = 0 would need a 33-bit step, so the host passes shift = 32,
// which selects the identity).
__device__ __forceinline__ uint32_t fast_div(uint32_t n, uint32_t mul, uint32_t shift)
{
    // a select, not a branch: a branch on a constant that was just loaded makes every caller
    // wait for that load before it may even request what it needs next
    const uint32_t t = __umulhi(mul, n);
    const uint32_t q = (t + ((n - t) >> 1)) >> (shift & 31);
    return shift == 32 ? n : q;
}

// Constants of fast_div for the divisor d >= 1.
inline void division_constants(uint32_t d, uint32_t& mul, uint32_t& shift)
{
    if (d == 1) {
        mul = 0;
        shift = 32;
        return;
    }
    uint32_t L = 0;
    while ((uint64_t{1} << L) < d)
        ++L;  // L = ceil(log2 d) >= 1
    mul = static_cast<uint32_t>(((uint64_t{1} << 32) * ((uint64_t{1} << L) - d)) / d + 1);
    shift = L - 1;
}

// Tuning and test options (dabnn_set_option in the C ABI; ids are the dabnn_option values).
// The library never reads the environment: an option has its default until a caller sets it.
int option(int id);

inline int device_cu_count()
{
    static const int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        return n;
    }();
    return cus;
}

// Resident workgroups of 256 threads per CU for a kernel (one wavefront per SIMD each), found
// once.  The runtime's occupancy query is the upper bound; measured on MI355X, wavefronts of
// launches sized by it alone start late when it answers 8, or 7 for a kernel with 65 to 72 vector
// registers: what is resident at once is at most 7 wavefronts per SIMD, with registers counted in
// blocks of 16.  A launch of exactly the resident size is what the balanced work splits assume.
template <class Kernel>
inline int resident_blocks_per_cu(Kernel kernel)
{
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kernel, 256, 0) != hipSuccess || nb <= 0)
        nb = 2;
    hipFuncAttributes attr;
    if (hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(kernel)) == hipSuccess && attr.numRegs > 0) {
        const int by_registers = 512 / ((attr.numRegs + 15) / 16 * 16);
        if (by_registers >= 1 && by_registers < nb)
            nb = by_registers;
    }
    return nb > 7 ? 7 : nb;
}

}  // namespace dabnn

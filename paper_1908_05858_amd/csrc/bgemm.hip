// BGEMM (Sec. 2.1.2, Eq. 1): C_ij = sum_k bitcount(xnor(A_ik, B_kj)) over bit-packed operands, and
// the patch-matrix (im2col) kernel that turns a convolution into such a product -- the route the
// paper compares its direct convolution with (Fig. 4).
//
// Operands are row-major packed matrices A [M][Kw] and B [N][Kw] (row j of B is the paper's
// column B_.j), Kw 64-bit words per row, of which the first K bits are real and the rest 0.
//
// "Row-stationary" kernel: lane l of a wavefront owns row 64*tile + l of A and keeps its 2*Kw
// dwords in VGPRs; the wavefront walks over groups of 16 rows of B, whose words are the same for
// every lane and therefore arrive through scalar loads and enter v_xor_b32 as the SGPR operand;
// v_bcnt_u32_b32 accumulates the popcount.  This is the activation-stationary convolution kernel
// with the window replaced by a matrix row; a 1x1 convolution is exactly this product.
#include "kernel_util.h"
#include "launch.h"

namespace dabnn {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

// acc[q] += popcount(w_q[0] ^ a0) + popcount(w_q[1] ^ a1) for four rows q of B.  w in SGPRs that
// only scalar loads write (see the note in bconv_areg.hip), a in VGPRs.
template <bool FIRST>
__device__ __forceinline__ void xor_popc_4x2(int* acc, uint32_t a0, uint32_t a1, const uint32_t* w0,
                                             const uint32_t* w1, const uint32_t* w2,
                                             const uint32_t* w3)
{
    uint32_t t0, t1, t2, t3;
#define DABNN_TAIL                        \
    "v_xor_b32 %4, %11, %9\n\t"           \
    "v_xor_b32 %5, %13, %9\n\t"           \
    "v_xor_b32 %6, %15, %9\n\t"           \
    "v_xor_b32 %7, %17, %9\n\t"           \
    "v_bcnt_u32_b32 %0, %4, %0\n\t"       \
    "v_bcnt_u32_b32 %1, %5, %1\n\t"       \
    "v_bcnt_u32_b32 %2, %6, %2\n\t"       \
    "v_bcnt_u32_b32 %3, %7, %3"
#define DABNN_HEAD                        \
    "v_xor_b32 %4, %10, %8\n\t"           \
    "v_xor_b32 %5, %12, %8\n\t"           \
    "v_xor_b32 %6, %14, %8\n\t"           \
    "v_xor_b32 %7, %16, %8\n\t"
#define DABNN_INPUTS                                                                             \
    "v"(a0), "v"(a1), "s"(w0[0]), "s"(w0[1]), "s"(w1[0]), "s"(w1[1]), "s"(w2[0]), "s"(w2[1]),     \
        "s"(w3[0]), "s"(w3[1])
    if constexpr (FIRST) {
        // the accumulators start here: the first popcounts add to the constant 0
        asm(DABNN_HEAD
            "v_bcnt_u32_b32 %0, %4, 0\n\t"
            "v_bcnt_u32_b32 %1, %5, 0\n\t"
            "v_bcnt_u32_b32 %2, %6, 0\n\t"
            "v_bcnt_u32_b32 %3, %7, 0\n\t" DABNN_TAIL
            : "=&v"(acc[0]), "=&v"(acc[1]), "=&v"(acc[2]), "=&v"(acc[3]), "=&v"(t0), "=&v"(t1),
              "=&v"(t2), "=&v"(t3)
            : DABNN_INPUTS);
    } else {
        asm(DABNN_HEAD
            "v_bcnt_u32_b32 %0, %4, %0\n\t"
            "v_bcnt_u32_b32 %1, %5, %1\n\t"
            "v_bcnt_u32_b32 %2, %6, %2\n\t"
            "v_bcnt_u32_b32 %3, %7, %3\n\t" DABNN_TAIL
            : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "=&v"(t0), "=&v"(t1),
              "=&v"(t2), "=&v"(t3)
            : DABNN_INPUTS);
    }
#undef DABNN_TAIL
#undef DABNN_HEAD
#undef DABNN_INPUTS
}

// A group = CG (16 or 32) rows of B against one 64-row tile of A.  Its scalar loads go through a
// double-buffered pipeline in units of CU rows of B x DU dwords (at most 24 SGPRs per buffer: two buffers plus the loop state must fit the SGPR file without spills).
template <int KD, int CGC>
struct GemmGeom {
    static constexpr int CG = CGC;
    static constexpr int DU = KD % 6 == 0 ? 6 : (KD % 4 == 0 ? 4 : 2);
    static constexpr int CU = DU == 2 ? 8 : 4;
    static constexpr int SB = CU * DU;
    static constexpr int CHUNKS = KD / DU;            // units per CU rows
    static constexpr int UNITS = (CG / CU) * CHUNKS;  // units per group (even)
};

template <int KD, int CGC, int UNIT, int SB>
__device__ __forceinline__ void gemm_load_unit(uint32_t (&sb)[SB], const uint32_t* __restrict__ b,
                                               int row0)
{
    using G = GemmGeom<KD, CGC>;
    constexpr int part = UNIT / G::CHUNKS;
    constexpr int chunk = UNIT % G::CHUNKS;
    const uint32_t* src = b + static_cast<size_t>(row0 + G::CU * part) * KD + chunk * G::DU;
#pragma unroll
    for (int q = 0; q < G::CU; ++q) {
#pragma unroll
        for (int d = 0; d < G::DU; ++d)
            sb[q * G::DU + d] = src[q * KD + d];
    }
}

template <int KD, int CGC, int UNIT, int SB>
__device__ __forceinline__ void gemm_compute_unit(const uint32_t (&sb)[SB], int (&acc)[CGC],
                                                  const uint32_t (&areg)[KD])
{
    using G = GemmGeom<KD, CGC>;
    constexpr int part = UNIT / G::CHUNKS;
    constexpr int chunk = UNIT % G::CHUNKS;
#pragma unroll
    for (int q4 = 0; q4 < G::CU; q4 += 4) {
        int* a4 = &acc[G::CU * part + q4];
        static_for<0, G::DU / 2>([&](auto dc) {
            constexpr int d = 2 * decltype(dc)::value;
            xor_popc_4x2<(chunk == 0 && d == 0)>(
                a4, areg[chunk * G::DU + d], areg[chunk * G::DU + d + 1], &sb[(q4 + 0) * G::DU + d],
                &sb[(q4 + 1) * G::DU + d], &sb[(q4 + 2) * G::DU + d], &sb[(q4 + 3) * G::DU + d]);
        });
    }
}

template <int KD, int CGC>
__global__ __launch_bounds__(256) void bgemm_rowreg_kernel(
    const uint32_t* __restrict__ A, const uint32_t* __restrict__ B, int32_t* __restrict__ C, int M,
    int N, int K, int neg_scale, int groups_per_tile, int n_ranges, int base_groups, int rem_groups)
{
    using G = GemmGeom<KD, CGC>;
    static_assert(G::UNITS % 2 == 0 && KD % G::DU == 0 && G::DU % 2 == 0, "pipeline geometry");
    __shared__ int32_t tile_lds[4 * 64 * CGC];  // 64 rows x CG columns of int32 per wavefront

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int gw = blockIdx.x * 4 + wave;
    if (gw >= n_ranges)
        return;  // the grid is rounded up to whole workgroups
    // balanced contiguous partition of (tile, group) pairs, group fastest
    int g = gw * base_groups + (gw < rem_groups ? gw : rem_groups);
    const int g_end = g + base_groups + (gw < rem_groups ? 1 : 0);
    if (g >= g_end)
        return;
    int tile = g / groups_per_tile;
    int cgi = g - tile * groups_per_tile;

    uint32_t areg[KD];
    auto load_rows = [&](int t) {
        const int r = min(t * 64 + lane, M - 1);  // rows past the end repeat the last one
        // uniform base + 32-bit byte offset (the launcher checks that the matrix fits)
        const char* src = reinterpret_cast<const char*>(A) + static_cast<uint32_t>(r) * (KD * 4u);
        if constexpr (KD % 4 == 0) {
#pragma unroll
            for (int d = 0; d < KD; d += 4) {
                const uint4 u = *reinterpret_cast<const uint4*>(src + d * 4);
                areg[d + 0] = u.x;
                areg[d + 1] = u.y;
                areg[d + 2] = u.z;
                areg[d + 3] = u.w;
            }
        } else {
#pragma unroll
            for (int d = 0; d < KD; d += 2) {
                const uint2 u = *reinterpret_cast<const uint2*>(src + d * 4);
                areg[d + 0] = u.x;
                areg[d + 1] = u.y;
            }
        }
    };
    load_rows(tile);

    uint32_t sb0[G::SB], sb1[G::SB];
    gemm_load_unit<KD, CGC, 0>(sb0, B, cgi * G::CG);

    for (; g < g_end; ++g) {
        int ncgi = cgi + 1, ntile = tile;
        if (ncgi == groups_per_tile) {
            ncgi = 0;
            ++ntile;
        }
        int acc[CGC];
        // Software pipeline: while unit u feeds the VALU, unit u+1 is in flight.
        static_for<0, G::UNITS>([&](auto uc) {
            constexpr int u = decltype(uc)::value;
            wait_scalar_loads();
            schedule_fence();
            if constexpr (u + 1 < G::UNITS) {
                if constexpr (u % 2 == 0)
                    gemm_load_unit<KD, CGC, u + 1>(sb1, B, cgi * G::CG);
                else
                    gemm_load_unit<KD, CGC, u + 1>(sb0, B, cgi * G::CG);
            } else {
                if (g + 1 < g_end)  // first unit of the next group (UNITS is even: buffer 0)
                    gemm_load_unit<KD, CGC, 0>(sb0, B, ncgi * G::CG);
            }
            schedule_fence();
            if constexpr (u % 2 == 0)
                gemm_compute_unit<KD, CGC, u>(sb0, acc, areg);
            else
                gemm_compute_unit<KD, CGC, u>(sb1, acc, areg);
            schedule_fence();
        });

        // Row P of the wavefront's LDS slice holds row P's CG results as QPR 16-byte quads; quad
        // j sits in column j ^ swz(P), which keeps both the row-wise writes and the transposed
        // reads free of bank conflicts (a 64-byte row covers half the banks, so two neighbouring
        // rows share one swizzle; a 128-byte row covers all of them).  QPR neighbouring lanes
        // then store the 64 or 128 contiguous bytes of one row of C, non-temporally: C is
        // written once and never read here.
        constexpr int QPR = CGC / 4;    // quads per row = lanes per row in the transposed store
        constexpr int PPI = 64 / QPR;   // rows per store instruction
        auto swz = [](int P) { return (CGC == 16) ? ((P >> 1) & 3) : (P & 7); };
        int32_t* slice = tile_lds + wave * (64 * CGC);
        {
            const int sw = swz(lane);
#pragma unroll
            for (int j = 0; j < QPR; ++j) {
                int4 o;
                // K - 2d (dot product) or K - d (match count), d < 2^23
                o.x = K + __mul24(neg_scale, acc[4 * j + 0]);
                o.y = K + __mul24(neg_scale, acc[4 * j + 1]);
                o.z = K + __mul24(neg_scale, acc[4 * j + 2]);
                o.w = K + __mul24(neg_scale, acc[4 * j + 3]);
                *reinterpret_cast<int4*>(slice + lane * CGC + 4 * (j ^ sw)) = o;
            }
        }
        // LDS instructions of one wavefront execute in order; this only stops the compiler from
        // moving the reads above the writes.
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int j = lane % QPR;
        char* dst = reinterpret_cast<char*>(C + static_cast<size_t>(tile) * 64 * N + cgi * G::CG);
#pragma unroll
        for (int k = 0; k < QPR; ++k) {
            const int P = PPI * k + lane / QPR;
            const int4 o = *reinterpret_cast<const int4*>(slice + P * CGC + 4 * (j ^ swz(P)));
            if (tile * 64 + P < M) {
                v4i v = {o.x, o.y, o.z, o.w};
                __builtin_nontemporal_store(
                    v, reinterpret_cast<v4i*>(dst + (static_cast<uint32_t>(P) * N + 4 * j) * 4u));
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();

        if (ntile != tile)
            load_rows(ntile);
        tile = ntile;
        cgi = ncgi;
    }
}

template <int KD, int CGC>
hipError_t launch_rowreg_cg(const uint32_t* A, const uint32_t* B, int32_t* C, int64_t M, int N, int K,
                            int mode, hipStream_t stream)
{
    auto kernel = bgemm_rowreg_kernel<KD, CGC>;
    static const int blocks_per_cu = resident_blocks_per_cu(kernel);
    const int64_t tiles = (M + 63) / 64;
    const int groups_per_tile = N / CGC;
    const int64_t n_groups64 = tiles * groups_per_tile;
    if (n_groups64 > 0x3fffffff)
        return hipErrorNotSupported;
    const int n_groups = static_cast<int>(n_groups64);
    // exactly the resident wavefront slots, every wavefront the same number of groups (+-1)
    int64_t ranges = static_cast<int64_t>(blocks_per_cu) * device_cu_count() * 4;
    if (ranges > n_groups)
        ranges = n_groups;
    const int n_ranges = static_cast<int>(ranges);
    const dim3 grid(static_cast<unsigned>((n_ranges + 3) / 4)), block(256);
    hipLaunchKernelGGL(kernel, grid, block, 0, stream, A, B, C, static_cast<int>(M), N, K,
                       mode == 1 ? -1 : -2, groups_per_tile, n_ranges, n_groups / n_ranges,
                       n_groups % n_ranges);
    return hipGetLastError();
}

template <int KD>
hipError_t launch_rowreg(const uint32_t* A, const uint32_t* B, int32_t* C, int64_t M, int N, int K,
                         int mode, hipStream_t stream)
{
    // With short rows the product is bound by the int32 output: 32 columns per group make every
    // store a whole 128-byte line.  Long rows keep 16 columns (fewer registers, finer work split).
    if constexpr (KD <= 16) {
        if (N % 32 == 0 && option(DABNN_OPT_BGEMM_COLUMNS) != 16)  // test hook: force 16 columns
            return launch_rowreg_cg<KD, 32>(A, B, C, M, N, K, mode, stream);
    }
    return launch_rowreg_cg<KD, 16>(A, B, C, M, N, K, mode, stream);
}

// ------------------------------------------------------------------------------ reference

// One thread per element of C; any shape.
__global__ __launch_bounds__(256) void bgemm_reference_kernel(
    const uint64_t* __restrict__ A, const uint64_t* __restrict__ B, int32_t* __restrict__ C,
    int64_t total, int N, int Kw, int K, int neg_scale)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (idx >= total)
        return;
    const int64_t i = idx / N;
    const int j = static_cast<int>(idx - i * N);
    const uint64_t* a = A + i * Kw;
    const uint64_t* b = B + static_cast<int64_t>(j) * Kw;
    int diff = 0;
    for (int q = 0; q < Kw; ++q)
        diff += __popcll(a[q] ^ b[q]);
    C[idx] = K + neg_scale * diff;
}

// ------------------------------------------------------------------------------ im2col

// One thread per word of the patch matrix [N*Ho*Wo][kh*kw][Cw]; a tap outside the image is an
// all-zero word (+1 in every channel), as in the convolution kernels.
__global__ __launch_bounds__(256) void im2col_kernel(const uint64_t* __restrict__ a,
                                                     uint64_t* __restrict__ cols, ConvShape s,
                                                     int64_t total)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (idx >= total)
        return;
    const int q = static_cast<int>(idx % s.Cw);
    int64_t t = idx / s.Cw;
    const int tap = static_cast<int>(t % (s.kh * s.kw));
    int64_t pix = t / (s.kh * s.kw);
    const int wo = static_cast<int>(pix % s.Wo);
    pix /= s.Wo;
    const int ho = static_cast<int>(pix % s.Ho);
    const int n = static_cast<int>(pix / s.Ho);
    const int hi = ho * s.stride - s.pad + tap / s.kw;
    const int wi = wo * s.stride - s.pad + tap % s.kw;
    uint64_t v = 0;
    if (hi >= 0 && hi < s.H && wi >= 0 && wi < s.W)
        v = a[((static_cast<int64_t>(n) * s.H + hi) * s.W + wi) * s.Cw + q];
    cols[idx] = v;
}

}  // namespace

bool bgemm_rowreg_supports(int64_t M, int N, int Kw, const void* C)
{
    switch (2 * Kw) {
        case 2: case 4: case 6: case 8: case 12: case 16: case 18: case 24: case 32: case 36:
        case 48: case 64: case 72: case 96: case 128: case 144:
            break;
        default:
            return false;
    }
    // 32-bit byte offsets into A and into a 64-row tile of C, 16-byte stores into C
    return N % 16 == 0 && M * Kw * 8 < (int64_t{1} << 32) &&
           static_cast<int64_t>(N) * 64 * 4 < (int64_t{1} << 32) &&
           (reinterpret_cast<uintptr_t>(C) & 15) == 0;
}

hipError_t launch_bgemm_rowreg(const uint64_t* A, const uint64_t* B, int32_t* C, int64_t M, int N,
                               int Kw, int K, int mode, hipStream_t stream)
{
    if (!bgemm_rowreg_supports(M, N, Kw, C))
        return hipErrorNotSupported;
    const uint32_t* a = reinterpret_cast<const uint32_t*>(A);
    const uint32_t* b = reinterpret_cast<const uint32_t*>(B);
    switch (2 * Kw) {
#define DABNN_CASE(KD) \
    case KD: return launch_rowreg<KD>(a, b, C, M, N, K, mode, stream);
        DABNN_CASE(2) DABNN_CASE(4) DABNN_CASE(6) DABNN_CASE(8) DABNN_CASE(12) DABNN_CASE(16)
        DABNN_CASE(18) DABNN_CASE(24) DABNN_CASE(32) DABNN_CASE(36) DABNN_CASE(48) DABNN_CASE(64)
        DABNN_CASE(72) DABNN_CASE(96) DABNN_CASE(128) DABNN_CASE(144)
#undef DABNN_CASE
        default: return hipErrorNotSupported;
    }
}

hipError_t launch_bgemm_reference(const uint64_t* A, const uint64_t* B, int32_t* C, int64_t M, int N,
                                  int Kw, int K, int mode, hipStream_t stream)
{
    const int64_t total = M * N;
    const int64_t blocks = (total + 255) / 256;
    bgemm_reference_kernel<<<dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream>>>(
        A, B, C, total, N, Kw, K, mode == 1 ? -1 : -2);
    return hipGetLastError();
}

hipError_t launch_im2col(const uint64_t* a, uint64_t* cols, const ConvShape& s, hipStream_t stream)
{
    const int64_t total = static_cast<int64_t>(s.N) * s.Ho * s.Wo * s.kh * s.kw * s.Cw;
    const int64_t blocks = (total + 255) / 256;
    im2col_kernel<<<dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream>>>(a, cols, s, total);
    return hipGetLastError();
}

}  // namespace dabnn

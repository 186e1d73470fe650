// Host-side sanitizer check of the library's dispatch code: built by tests/test_oracle_sanitize.py
// from csrc/dabnn_api.hip (host side instrumented with -fsanitize=address,undefined) plus the
// library's other object files, and run WITHOUT a GPU: every call below must be refused on the
// host or computed there (dabnn_bn_thresholds, dabnn_bconv2d_pick_algo, the options).  Host
// buffers have exactly their size, so a write past either end is reported.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/dabnn.h"

#define CHECK(cond)                                                      \
    do {                                                                 \
        if (!(cond)) {                                                   \
            std::printf("check failed at line %d: %s\n", __LINE__, #cond); \
            return 1;                                                    \
        }                                                                \
    } while (0)

int main()
{
    auto* a = reinterpret_cast<uint64_t*>(0x10000);
    auto* w = reinterpret_cast<uint64_t*>(0x20000);
    auto* y = reinterpret_cast<int32_t*>(0x30000);
    CHECK(dabnn_bconv2d(a, w, y, 1, 4, 4, 64, 64, 3, 3, 1, 3, nullptr) == DABNN_ERR_SHAPE);
    CHECK(dabnn_bconv2d(a, w, y, INT32_MAX, 1 << 15, 1 << 15, 64, 64, 3, 3, 1, 1, nullptr) == DABNN_ERR_SHAPE);
    CHECK(dabnn_bconv2d(a, w, reinterpret_cast<int32_t*>(0x30002), 1, 4, 4, 64, 64, 3, 3, 1, 1, nullptr) ==
          DABNN_ERR_ALIGN);
    CHECK(dabnn_bconv2d(nullptr, w, y, 1, 4, 4, 64, 64, 3, 3, 1, 1, nullptr) == DABNN_ERR_NULL);
    CHECK(dabnn_bconv2d_algo(a, w, y, 1, 4, 4, 64, 8, 3, 3, 1, 1, 9, nullptr) == DABNN_ERR_UNSUPPORTED);
    const int shapes[][9] = {{256, 56, 56, 64, 64, 3, 3, 1, 1},   {1, 7, 7, 512, 512, 3, 3, 2, 1},
                             {3, 9, 9, 100, 7, 5, 5, 3, 2},       {2, 6, 6, 128, 64, 1, 1, 1, 0},
                             {1, 8200, 8200, 512, 16, 3, 3, 1, 1}, {4, 14, 14, 320, 64, 3, 3, 1, 1},
                             {2, 14, 14, 1024, 128, 3, 3, 2, 1}};
    for (const auto& s : shapes) {
        const int algo = dabnn_bconv2d_pick_algo(s[0], s[1], s[2], s[3], s[4], s[5], s[6], s[7], s[8]);
        CHECK(algo >= DABNN_ALGO_REFERENCE && algo <= DABNN_ALGO_BGEMM);
    }
    CHECK(dabnn_bconv2d_pick_algo(1, 56, 56, 64, 64, 3, 3, 0, 1) == -1);
    CHECK(dabnn_bgemm(a, w, y, int64_t{1} << 40, 16, 1, 64, 0, nullptr) == DABNN_ERR_SHAPE);
    CHECK(dabnn_bitpack(reinterpret_cast<const float*>(a), w, int64_t{1} << 41, 1 << 10, 0, nullptr) ==
          DABNN_ERR_SHAPE);
    CHECK(dabnn_im2col(a, w, 1 << 10, 1 << 10, 1 << 10, 64, 3, 3, 1, 1, nullptr) == DABNN_ERR_SHAPE);
    CHECK(dabnn_expand_int8(a, reinterpret_cast<int8_t*>(y), 4, 80, nullptr) == DABNN_ERR_UNSUPPORTED);
    CHECK(dabnn_set_option(DABNN_OPT_COUNT, 1) == DABNN_ERR_UNSUPPORTED);
    CHECK(dabnn_set_option(-1, 1) == DABNN_ERR_UNSUPPORTED);
    CHECK(dabnn_set_option(DABNN_OPT_AREG_STORE, 16) == DABNN_OK && dabnn_get_option(DABNN_OPT_AREG_STORE) == 16);
    CHECK(dabnn_set_option(DABNN_OPT_AREG_STORE, 0) == DABNN_OK && dabnn_get_option(DABNN_OPT_COUNT) == -1);

    // dabnn_bn_thresholds writes thr[Cout] and flip[ceil(Cout/64)]: exact-size buffers, awkward
    // parameters (zeros, denormal and huge scales, zero and huge variances)
    for (int C : {1, 63, 64, 65, 300}) {
        const int K = 4608;
        std::vector<float> g(C), b(C), m(C), v(C);
        unsigned st = 99u + C;
        auto rnd = [&]() { st = st * 1664525u + 1013904223u; return (st >> 8) / 16777216.0f; };
        for (int c = 0; c < C; ++c) {
            g[c] = 6.0f * rnd() - 3.0f;
            b[c] = 4.0f * rnd() - 2.0f;
            m[c] = 1000.0f * rnd() - 500.0f;
            v[c] = 50.0f * rnd();
        }
        g[0] = 0.0f;
        if (C > 8) {
            g[1] = 1e-38f; g[2] = -3e38f; b[3] = 3e38f; b[4] = -3e38f; m[6] = 3e38f; v[7] = 0.0f; v[8] = 3e38f;
        }
        std::vector<int32_t> thr(C);
        std::vector<uint64_t> flip((C + 63) / 64);
        CHECK(dabnn_bn_thresholds(g.data(), b.data(), m.data(), v.data(), 1e-5f, C, K, thr.data(),
                                  flip.data()) == DABNN_OK);
        for (int c = 0; c < C; ++c)
            CHECK(thr[c] >= -(1 << 30) && thr[c] <= (1 << 30));
        if (C % 64)
            CHECK((flip.back() >> (C % 64)) == 0);
    }
    std::puts("host dispatch sanitizer run ok");
    return 0;
}

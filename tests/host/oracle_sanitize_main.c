/* Host-side sanitizer check of the oracle: built with -fsanitize=address,undefined
 * -fno-sanitize-recover by tests/test_oracle_sanitize.py together with oracle/dabnn_oracle.c and
 * run on small, awkward shapes (tails, borders wider than the image, strides above the pad), every
 * buffer allocated at exactly its size so that an access past either end is reported.  It exits 0
 * when no check fires; results are not compared here (the pins do that). */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_sign(const float *x, float *s, int64_t n, int rule);
int oracle_bitpack(const float *x, uint64_t *out, int64_t n_pixels, int C, int rule);
int oracle_bitpack_i32(const int32_t *x, uint64_t *out, int64_t n_pixels, int C);
int oracle_bconv2d(const float *A, const float *Wt, int32_t *Y, int N, int H, int W, int Cin,
                   int Cout, int kh, int kw, int stride, int pad);
int oracle_bconv2d_zeropad(const float *A, const float *Wt, int32_t *Y, int N, int H, int W,
                           int Cin, int Cout, int kh, int kw, int stride, int pad);
int oracle_bgemm(const float *A, const float *B, int32_t *C, int64_t M, int N, int K, int mode);
int oracle_bn_sign_pack(const int32_t *y, const float *scale, const float *shift, const float *r,
                        float *x_out, uint64_t *bits, int64_t n_pixels, int C);
int oracle_nhwc_to_nc1hwc2(const uint64_t *in, uint64_t *out, int N, int H, int W, int Cw);
int oracle_bconv2d_at(const float *A, const float *Wt, const int32_t *idx, int64_t n_samples,
                      int32_t *out, int N, int H, int W, int Cin, int Cout, int kh, int kw,
                      int stride, int pad);
int oracle_bconv2d_bnsign(const float *A, const float *Wt, const float *gamma, const float *beta,
                          const float *mean, const float *var, float eps, uint64_t *out, int N,
                          int H, int W, int Cin, int Cout, int kh, int kw, int stride, int pad);
int oracle_glue(const float *x, const int32_t *y, const float *gamma, const float *beta,
                float *x_next, int N, int H, int W, int Cin, int Ho, int Wo, int Cout, int K,
                int stride);

static float pm1(unsigned *st)
{
    *st = *st * 1664525u + 1013904223u;
    return (*st >> 16) & 1 ? 1.0f : -1.0f;
}

int main(void)
{
    const int shapes[][8] = {{1, 1, 1, 1, 1, 3, 1, 1}, {2, 5, 4, 70, 3, 3, 2, 1},
                             {1, 2, 9, 64, 5, 5, 1, 2}, {1, 6, 6, 130, 2, 1, 3, 0}};
    unsigned st = 12345u;
    for (unsigned t = 0; t < sizeof shapes / sizeof shapes[0]; ++t) {
        const int N = shapes[t][0], H = shapes[t][1], W = shapes[t][2], Cin = shapes[t][3],
                  Cout = shapes[t][4], k = shapes[t][5], s = shapes[t][6], p = shapes[t][7];
        const int Ho = (H + 2 * p - k) / s + 1, Wo = (W + 2 * p - k) / s + 1;
        const int64_t na = (int64_t)N * H * W * Cin, nw = (int64_t)Cout * k * k * Cin;
        const int64_t ny = (int64_t)N * Ho * Wo * Cout;
        float *A = malloc(sizeof(float) * na), *Wt = malloc(sizeof(float) * nw);
        int32_t *Y = malloc(sizeof(int32_t) * ny);
        uint64_t *bits = malloc(8 * (size_t)(na / Cin) * ((Cin + 63) / 64));
        for (int64_t i = 0; i < na; ++i) A[i] = pm1(&st);
        for (int64_t i = 0; i < nw; ++i) Wt[i] = pm1(&st);
        if (oracle_sign(A, A, na, 0) || oracle_bitpack(A, bits, na / Cin, Cin, 1) ||
            oracle_bconv2d(A, Wt, Y, N, H, W, Cin, Cout, k, k, s, p) ||
            oracle_bconv2d_zeropad(A, Wt, Y, N, H, W, Cin, Cout, k, k, s, p) ||
            oracle_bgemm(A, Wt, Y, 1, 1, Cin, 1) || oracle_bitpack_i32(Y, bits, 1, 1))
            return 2;
        float *sc = malloc(sizeof(float) * Cout), *z = malloc(sizeof(float) * ny);
        uint64_t *ob = malloc(8 * (size_t)(ny / Cout) * ((Cout + 63) / 64));
        for (int c = 0; c < Cout; ++c) sc[c] = 0.01f * (float)(c - 1);
        if (oracle_bn_sign_pack(Y, sc, sc, z, z, ob, ny / Cout, Cout))
            return 3;
        /* the last output, one by one; the fused batch-norm + sign; both into exact-size buffers */
        int32_t idx[4] = {N - 1, Ho - 1, Wo - 1, Cout - 1}, one;
        if (oracle_bconv2d_at(A, Wt, idx, 1, &one, N, H, W, Cin, Cout, k, k, s, p))
            return 5;
        if (oracle_bconv2d_bnsign(A, Wt, sc, sc, sc, sc, 1e-5f, ob, N, H, W, Cin, Cout, k, k, s, p))
            return 6;
        free(A); free(Wt); free(Y); free(bits); free(sc); free(z); free(ob);
    }
    uint64_t in[2 * 3 * 3], out[2 * 2 * 3 * 2];
    for (int i = 0; i < 18; ++i) in[i] = (uint64_t)i * 0x9e3779b97f4a7c15ull;
    if (oracle_nhwc_to_nc1hwc2(in, out, 2, 1, 3, 3))
        return 4;
    /* the input generator of the full-network workload: stride 1 (identity shortcut) and stride 2
     * (2x2 mean clipped at an odd edge, channels repeated) */
    {
        enum { N = 2, H = 5, W = 3, C = 3 };
        float x[N * H * W * C], g[2 * C], b[2 * C];
        int32_t y1[N * H * W * C], y2[N * 3 * 2 * 2 * C];
        float o1[N * H * W * C], o2[N * 3 * 2 * 2 * C];
        for (int i = 0; i < N * H * W * C; ++i) { x[i] = pm1(&st); y1[i] = i - 40; }
        for (int i = 0; i < N * 3 * 2 * 2 * C; ++i) y2[i] = 7 - i;
        for (int i = 0; i < 2 * C; ++i) { g[i] = 1.0f + i; b[i] = -0.5f * i; }
        if (oracle_glue(x, y1, g, b, o1, N, H, W, C, H, W, C, 27, 1) ||
            oracle_glue(x, y2, g, b, o2, N, H, W, C, 3, 2, 2 * C, 27, 2))
            return 7;
    }
    puts("oracle sanitizer run ok");
    return 0;
}

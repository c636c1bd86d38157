/* Runs every function of oracle/int8t_oracle.c on small inputs (ragged sizes, padding, strides,
 * depthwise, empty tensors) in a build with -fsanitize=address,undefined: an access outside a
 * buffer, a signed overflow or a bad shift inside the oracle stops the program.  The oracle source
 * is #included so that its static helpers are instrumented too.  Prints "oracle sanitize ok". */
#include "../../oracle/int8t_oracle.c"

#include <stdio.h>

static uint32_t lcg(uint32_t *s) { *s = *s * 1664525u + 1013904223u; return *s >> 8; }

static int run_layer(int N, int C, int H, int W, int K, int R, int S, int sh, int sw, int ph, int pw, int g)
{
    orc_conv_desc d = {N, C, H, W, K, R, S, sh, sw, ph, pw, g};
    const int P = orc_out_h(&d), Q = orc_out_w(&d);
    if (P < 1 || Q < 1) return 0;
    const size_t nx = (size_t)N * C * H * W, nw = (size_t)K * (C / g) * R * S, ny = (size_t)N * K * P * Q;
    int8_t *x = malloc(nx), *w = malloc(nw), *dy = malloc(ny);
    int64_t *y = malloc(ny * 8), *dx = malloc(nx * 8), *dw = malloc(nw * 8);
    uint32_t s = 12345u + (uint32_t)(N * 7 + C * 3 + R);
    for (size_t i = 0; i < nx; ++i) x[i] = (int8_t)((int)(lcg(&s) % 255u) - 127);
    for (size_t i = 0; i < nw; ++i) w[i] = (int8_t)((int)(lcg(&s) % 255u) - 127);
    for (size_t i = 0; i < ny; ++i) dy[i] = (int8_t)((int)(lcg(&s) % 255u) - 127);
    orc_conv_fwd(&d, x, w, y);
    orc_conv_bwd_data(&d, dy, w, dx);
    orc_conv_bwd_weight(&d, x, dy, dw);
    /* the single-output forms must agree with the whole-tensor forms at the corners */
    int bad = 0;
    bad += y[0] != orc_conv_fwd_at(&d, x, w, 0, 0, 0, 0);
    bad += y[ny - 1] != orc_conv_fwd_at(&d, x, w, N - 1, K - 1, P - 1, Q - 1);
    bad += dx[nx - 1] != orc_conv_bwd_data_at(&d, dy, w, N - 1, C - 1, H - 1, W - 1);
    bad += dw[nw - 1] != orc_conv_bwd_weight_at(&d, x, dy, K - 1, C / g - 1, R - 1, S - 1);
    /* exact adjoint identity */
    int64_t a = 0, b = 0, c = 0;
    for (size_t i = 0; i < ny; ++i) a += (int64_t)dy[i] * y[i];
    for (size_t i = 0; i < nx; ++i) b += (int64_t)x[i] * dx[i];
    for (size_t i = 0; i < nw; ++i) c += (int64_t)w[i] * dw[i];
    bad += (a != b) + (a != c);
    int32_t *y32 = malloc(ny * 4);
    float *yf = malloc(ny * 4);
    int64_t ov = 0;
    orc_wrap32(y, ny, y32, &ov);
    orc_dequant(y32, ny, 0.01f, 0.002f, yf);
    free(x); free(w); free(dy); free(y); free(dx); free(dw); free(y32); free(yf);
    return bad;
}

int main(void)
{
    int bad = 0;
    /* quantizers and clip search: lengths 0, 1, ragged; both modes; zero tensor; huge and tiny values */
    const size_t sizes[] = {0, 1, 3, 257, 5000};
    for (unsigned k = 0; k < sizeof(sizes) / sizeof(sizes[0]); ++k) {
        const size_t n = sizes[k];
        float *g = malloc((n ? n : 1) * sizeof(float));
        int8_t *q = malloc(n ? n : 1);
        uint32_t s = 99u + (uint32_t)n;
        for (size_t i = 0; i < n; ++i) g[i] = ((float)(lcg(&s) % 2001u) - 1000.0f) * 1e-4f * (i % 97 == 0 ? 100.0f : 1.0f);
        if (n > 2) { g[1] = 3.0e38f; g[2] = -1.0e-40f; }
        const float m = orc_absmax(g, n);
        for (int mode = 0; mode < 2; ++mode) {
            float sc = -1.0f;
            orc_quantize(g, n, m, mode, 0x123456789ABCULL, q, &sc);
            const double d = orc_deviation(g, q, sc, n);
            bad += !(d >= -1e-12 && d <= 2.0 + 1e-12);
            orc_quantize(g, n, 0.0f, mode, 7, q, &sc);
            for (size_t i = 0; i < n; ++i) bad += q[i] != 0;
            float ratios[5] = {1.0f, 0.5f, 0.25f, 0.01f, 1e-6f}, clips[5];
            double dev[5];
            int js = -1;
            orc_dsgc(g, n, ratios, 5, mode, 42, clips, dev, &js);
            bad += js < 0 || js > 4;
        }
        free(g);
        free(q);
    }
    bad += orc_rng24(~0ULL, ~0ULL) >= (1u << 24);
    bad += !(orc_dclr(0.0, 20.0, 0.1) == 1.0) + !(orc_dclr(2.0, 20.0, 0.1) == 0.1);
    bad += !(orc_scale(127.0f) == 1.0f) + !(orc_scale(0.0f) == 0.0f);
    /* convolutions */
    bad += run_layer(2, 3, 5, 7, 4, 3, 3, 1, 1, 1, 1, 1);
    bad += run_layer(1, 5, 9, 8, 6, 1, 7, 1, 1, 0, 3, 1);
    bad += run_layer(2, 4, 11, 6, 3, 7, 1, 2, 1, 3, 0, 1);
    bad += run_layer(1, 6, 10, 10, 6, 5, 5, 3, 2, 2, 2, 6);
    bad += run_layer(3, 2, 4, 4, 5, 2, 2, 3, 3, 0, 0, 1);
    bad += run_layer(1, 1, 1, 1, 1, 1, 1, 1, 1, 0, 0, 1);
    if (bad) {
        printf("oracle sanitize: %d checks failed\n", bad);
        return 1;
    }
    printf("oracle sanitize ok\n");
    return 0;
}

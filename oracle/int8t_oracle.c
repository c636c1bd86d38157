/*
 * int8t oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, obviously-correct CPU statement of what the INT8 training
 * convolution path of "Towards Unified INT8 Training for Convolutional Neural
 * Network" computes.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.  It shares no code, header, table or constant
 * generator with the GPU library; it is written from the paper's definitions:
 *
 *   Eq.1  symmetric uniform quantizer   q = round(clip(x,c)/s), s = c/(2^7-1)
 *   Eq.2  dequantize                    xhat = q*s
 *   Eq.3  stochastic rounding           floor(x) w.p. 1-frac, floor(x)+1 w.p. frac
 *   Eq.6  direction deviation           d_c = 1 - g.ghat / (|g| |ghat|)
 *   Eq.7  LR scaling                    phi(d_c) = max(exp(-alpha d_c), beta)
 *   Sec.3.4  g_W = g_z^T a, only g_z is (stochastically) quantized
 *   Suppl. "INT8 Convolution": int8 x int8 products accumulated in 32 bits
 *
 * Floating point is fp32 exactly where the method's *decisions* are taken in
 * fp32 (the scaled value t whose rounding gives the int8 code) and double /
 * int64 everywhere else.  Build with -ffp-contract=off (no fused multiply-add)
 * so that every fp32 operation below rounds once, as written.
 *
 * Parity pins (tests/test_oracle_*.py): every function here is pinned by
 * closed forms, invariants, library cross-checks or brute force, except the
 * absolute value of d_c on the paper's *real* gradients, which needs the
 * paper's training runs: "parity unpinned" for that quantity only.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* absmax: upper end of the clip range, max(|l|,|u|)  (Sec.3.1, text   */
/* before Eq.1).  NaNs are ignored (fmaxf semantics).                  */
/* ------------------------------------------------------------------ */
float orc_absmax(const float *x, size_t n)
{
    float m = 0.0f;
    for (size_t i = 0; i < n; ++i) {
        float a = fabsf(x[i]);
        if (a > m) m = a;
    }
    return m;
}

/* ------------------------------------------------------------------ */
/* Counter-based uniform draw for Eq.3.  The paper's generator (Eq.8,  */
/* an LCG seeded from the first datum plus the thread index) depends   */
/* on launch geometry and does not print its constants, so it cannot   */
/* be reproduced; it is replaced by a stateless function of            */
/* (seed, logical element index) returning 24 uniform bits.            */
/* Reading: a 32-bit avalanche finaliser (multiply / xor-shift, the    */
/* published murmur3 finaliser constants) applied to (index ^ kx) + ka, */
/* where the two 32-bit keys come from the 64-bit seed through the     */
/* same finaliser:  kx = mix(low ^ mix(high + 0x9E3779B9)),            */
/* ka = mix(kx + 0x9E3779B9).  For a fixed seed this is a bijection of */
/* the 32-bit index, hence exactly equidistributed over a full period; */
/* hashing the seed first keeps the tables of related seeds (1, 2, 3,  */
/* ... as a training loop hands them out) from being xor-shifted       */
/* copies of each other.                                               */
/* ------------------------------------------------------------------ */
static uint32_t orc_mix32(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x85EBCA6Bu;
    x ^= x >> 13;
    x *= 0xC2B2AE35u;
    x ^= x >> 16;
    return x;
}

uint32_t orc_rng24(uint64_t seed, uint64_t index)
{
    uint32_t lo = (uint32_t)(seed & 0xFFFFFFFFu);
    uint32_t hi = (uint32_t)(seed >> 32);
    uint32_t kx = orc_mix32(lo ^ orc_mix32(hi + 0x9E3779B9u));
    uint32_t ka = orc_mix32(kx + 0x9E3779B9u);
    return orc_mix32(((uint32_t)index ^ kx) + ka) >> 8;
}

/* ------------------------------------------------------------------ */
/* Eq.1 / Eq.3 for one element.                                        */
/*   inv = 127/c          one fp32 division (= 1/s)                    */
/*   mode 0: t = clip(x*inv, 127) in fp32; clip(x,c)/s == clip(x/s,    */
/*         127) for s > 0, evaluated on the scaled value so that       */
/*         |t| <= 127 holds exactly and codes never leave [-127,127];  */
/*         q = rint(t), ties to even                                   */
/*   mode 1: Eq.3 with 24-bit probabilities, applied to the magnitude  */
/*         and the sign restored (floor(t) and floor(t)+1 keep exactly */
/*         the probabilities of Eq.3, also for negative t):            */
/*         P = |x| * (inv*2^24)      exact real product (both factors  */
/*             are fp32, so it fits a double; inv*2^24 is an exact     */
/*             power-of-two scaling of inv)                            */
/*         m = min(127, floor((P + u) / 2^24)),  u = rng24(seed,index) */
/*         q = sign(x) * m                                             */
/*         => |q| = floor(|t|)+1 with probability frac(|t|), resolved  */
/*            to 2^-24; integer t are fixed points                     */
/* c <= 0 (all-zero tensor): every code is 0.  NaN -> code 0.          */
/* ------------------------------------------------------------------ */
static inline float orc_inv_scale(float c)
{
    return (c > 0.0f) ? (127.0f / c) : 0.0f;
}

static inline int orc_quantize_one(float x, float inv, int mode, uint64_t seed, uint64_t index)
{
    if (mode == 0) {
        float t = x * inv;
        if (t > 127.0f) t = 127.0f;
        if (t < -127.0f) t = -127.0f;
        if (t != t) t = 0.0f;
        return (int)rintf(t); /* default rounding mode: nearest, ties to even */
    } else {
        float inv24 = inv * 16777216.0f;
        double P = (double)fabsf(x) * (double)inv24; /* exact: 24 x 24 significant bits */
        int m;
        if (P != P) {
            m = 0; /* NaN input, or 0 * inf */
        } else if (P >= 2147483648.0) {
            m = 127;
        } else {
            int64_t S = (int64_t)floor(P) + (int64_t)orc_rng24(seed, index); /* floor(P + u), u integer */
            m = (S >= 2147483648LL) ? 127 : (int)(S >> 24);
        }
        return (x < 0.0f) ? -m : m;
    }
}

/* scale factor s = c / (2^(8-1) - 1)   (text after Eq.1) */
float orc_scale(float c)
{
    return (c > 0.0f) ? (c / 127.0f) : 0.0f;
}

/* Quantize a whole tensor in logical (row-major) element order. */
void orc_quantize(const float *x, size_t n, float c, int mode, uint64_t seed,
                  int8_t *q, float *scale_out)
{
    float inv = orc_inv_scale(c);
    for (size_t i = 0; i < n; ++i)
        q[i] = (int8_t)orc_quantize_one(x[i], inv, mode, seed, (uint64_t)i);
    if (scale_out) *scale_out = orc_scale(c);
}

/* ------------------------------------------------------------------ */
/* Eq.6, literally: ghat_i = q_i * s (Eq.2), then                      */
/* d = 1 - (sum g ghat) / (sqrt(sum g^2) * sqrt(sum ghat^2)),          */
/* sequential double sums.  Degenerate cases (the paper is silent):    */
/* |g| = 0 -> d = 0 (nothing to deviate from); |ghat| = 0 with         */
/* |g| > 0 -> d = 1 (no direction kept).                               */
/* ------------------------------------------------------------------ */
double orc_deviation(const float *g, const int8_t *q, float s, size_t n)
{
    double sgh = 0.0, sgg = 0.0, shh = 0.0;
    for (size_t i = 0; i < n; ++i) {
        double gi = (double)g[i];
        double hi = (double)q[i] * (double)s;
        sgh += gi * hi;
        sgg += gi * gi;
        shh += hi * hi;
    }
    if (sgg == 0.0) return 0.0;
    if (shh == 0.0) return 1.0;
    return 1.0 - sgh / (sqrt(sgg) * sqrt(shh));
}

/* ------------------------------------------------------------------ */
/* Direction Sensitive Gradient Clipping (Sec.3.4) as a brute-force    */
/* candidate search: for each candidate clip c_j = fl32(absmax *       */
/* ratio_j) quantize the whole tensor (same mode, same draws as the    */
/* real quantization), dequantize, evaluate Eq.6, keep the smallest    */
/* deviation; exact ties go to the smallest j.                         */
/* Outputs: clips[J], dev[J], *jstar.  Returns absmax.                 */
/* ------------------------------------------------------------------ */
float orc_dsgc(const float *g, size_t n, const float *ratios, int J, int mode,
               uint64_t seed, float *clips, double *dev, int *jstar)
{
    float m = orc_absmax(g, n);
    int8_t *q = (int8_t *)malloc(n ? n : 1);
    int best = 0;
    for (int j = 0; j < J; ++j) {
        float c = m * ratios[j];
        float s;
        orc_quantize(g, n, c, mode, seed, q, &s);
        clips[j] = c;
        dev[j] = orc_deviation(g, q, s, n);
        if (dev[j] < dev[best]) best = j;
    }
    free(q);
    if (m == 0.0f) best = 0;
    *jstar = best;
    return m;
}

/* Eq.7 */
double orc_dclr(double d, double alpha, double beta)
{
    double e = exp(-alpha * d);
    return (e > beta) ? e : beta;
}

/* ------------------------------------------------------------------ */
/* Convolutions on int8 codes, exact in int64.  PyTorch conventions:   */
/* cross-correlation, x[N][C][H][W], w[K][C/g][R][S], y[N][K][P][Q],   */
/* zero padding, P = floor((H + 2 pad_h - R)/stride_h) + 1, dilation 1.*/
/* Each of the three is written as its own gather sum; none is derived */
/* from another.                                                       */
/* ------------------------------------------------------------------ */
typedef struct {
    int N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups;
} orc_conv_desc;

int orc_out_h(const orc_conv_desc *d) { return (d->H + 2 * d->pad_h - d->R) / d->stride_h + 1; }
int orc_out_w(const orc_conv_desc *d) { return (d->W + 2 * d->pad_w - d->S) / d->stride_w + 1; }

/* forward: z[n,k,p,q] = sum_{c,r,s} a[n, c, p*sh + r - ph, q*sw + s - pw] * W[k,c,r,s] */
int64_t orc_conv_fwd_at(const orc_conv_desc *d, const int8_t *x, const int8_t *w,
                        int n, int k, int p, int q)
{
    int Cg = d->C / d->groups, Kg = d->K / d->groups;
    int g = k / Kg;
    int64_t acc = 0;
    for (int c = 0; c < Cg; ++c)
        for (int r = 0; r < d->R; ++r)
            for (int s = 0; s < d->S; ++s) {
                int h = p * d->stride_h + r - d->pad_h;
                int ww = q * d->stride_w + s - d->pad_w;
                if (h < 0 || h >= d->H || ww < 0 || ww >= d->W) continue;
                int64_t xv = x[(((size_t)n * d->C + (size_t)(g * Cg + c)) * d->H + h) * d->W + ww];
                int64_t wv = w[(((size_t)k * Cg + c) * d->R + r) * d->S + s];
                acc += xv * wv;
            }
    return acc;
}

void orc_conv_fwd(const orc_conv_desc *d, const int8_t *x, const int8_t *w, int64_t *acc)
{
    int P = orc_out_h(d), Q = orc_out_w(d);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < d->N; ++n)
        for (int k = 0; k < d->K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q)
                    acc[(((size_t)n * d->K + k) * P + p) * Q + q] = orc_conv_fwd_at(d, x, w, n, k, p, q);
}

/* backward-data: g_a[n,c,h,w] = sum_{k,r,s} g_z[n,k,p,q] * W[k,c,r,s]
 * over those (p,q) with p*sh + r - ph = h and q*sw + s - pw = w. */
int64_t orc_conv_bwd_data_at(const orc_conv_desc *d, const int8_t *dy, const int8_t *w,
                             int n, int c, int h, int ww)
{
    int P = orc_out_h(d), Q = orc_out_w(d);
    int Cg = d->C / d->groups, Kg = d->K / d->groups;
    int g = c / Cg, cl = c - g * Cg;
    int64_t acc = 0;
    for (int kk = 0; kk < Kg; ++kk) {
        int k = g * Kg + kk;
        for (int r = 0; r < d->R; ++r) {
            int th = h + d->pad_h - r;
            if (th < 0 || th % d->stride_h != 0) continue;
            int p = th / d->stride_h;
            if (p >= P) continue;
            for (int s = 0; s < d->S; ++s) {
                int tw = ww + d->pad_w - s;
                if (tw < 0 || tw % d->stride_w != 0) continue;
                int q = tw / d->stride_w;
                if (q >= Q) continue;
                int64_t gv = dy[(((size_t)n * d->K + k) * P + p) * Q + q];
                int64_t wv = w[(((size_t)k * Cg + cl) * d->R + r) * d->S + s];
                acc += gv * wv;
            }
        }
    }
    return acc;
}

void orc_conv_bwd_data(const orc_conv_desc *d, const int8_t *dy, const int8_t *w, int64_t *acc)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < d->N; ++n)
        for (int c = 0; c < d->C; ++c)
            for (int h = 0; h < d->H; ++h)
                for (int ww = 0; ww < d->W; ++ww)
                    acc[(((size_t)n * d->C + c) * d->H + h) * d->W + ww] =
                        orc_conv_bwd_data_at(d, dy, w, n, c, h, ww);
}

/* backward-weight: g_W[k,c,r,s] = sum_{n,p,q} g_z[n,k,p,q] * a[n, c, p*sh + r - ph, q*sw + s - pw] */
int64_t orc_conv_bwd_weight_at(const orc_conv_desc *d, const int8_t *x, const int8_t *dy,
                               int k, int c, int r, int s)
{
    int P = orc_out_h(d), Q = orc_out_w(d);
    int Cg = d->C / d->groups, Kg = d->K / d->groups;
    int g = k / Kg;
    int64_t acc = 0;
    for (int n = 0; n < d->N; ++n)
        for (int p = 0; p < P; ++p) {
            int h = p * d->stride_h + r - d->pad_h;
            if (h < 0 || h >= d->H) continue;
            for (int q = 0; q < Q; ++q) {
                int ww = q * d->stride_w + s - d->pad_w;
                if (ww < 0 || ww >= d->W) continue;
                int64_t gv = dy[(((size_t)n * d->K + k) * P + p) * Q + q];
                int64_t xv = x[(((size_t)n * d->C + (size_t)(g * Cg + c)) * d->H + h) * d->W + ww];
                acc += gv * xv;
            }
        }
    return acc;
}

void orc_conv_bwd_weight(const orc_conv_desc *d, const int8_t *x, const int8_t *dy, int64_t *acc)
{
    int Cg = d->C / d->groups;
#pragma omp parallel for collapse(2) schedule(static)
    for (int k = 0; k < d->K; ++k)
        for (int c = 0; c < Cg; ++c)
            for (int r = 0; r < d->R; ++r)
                for (int s = 0; s < d->S; ++s)
                    acc[(((size_t)k * Cg + c) * d->R + r) * d->S + s] =
                        orc_conv_bwd_weight_at(d, x, dy, k, c, r, s);
}

/* ------------------------------------------------------------------ */
/* 32-bit accumulator view and Eq.2 epilogue.  The hardware sums in    */
/* 32 bits (two's complement wrap); the compared integer is the low 32 */
/* bits of the exact sum, and *overflow counts sums outside int32.     */
/* Dequantized value: wrapped_acc * s_a * s_b in double, rounded once  */
/* to fp32.                                                            */
/* ------------------------------------------------------------------ */
void orc_wrap32(const int64_t *acc, size_t n, int32_t *out, int64_t *overflow)
{
    int64_t ov = 0;
    for (size_t i = 0; i < n; ++i) {
        int64_t a = acc[i];
        if (a > 2147483647LL || a < -2147483648LL) ++ov;
        out[i] = (int32_t)(uint32_t)((uint64_t)a & 0xFFFFFFFFu);
    }
    if (overflow) *overflow = ov;
}

void orc_dequant(const int32_t *acc, size_t n, float sa, float sb, float *out)
{
    for (size_t i = 0; i < n; ++i)
        out[i] = (float)((double)acc[i] * (double)sa * (double)sb);
}

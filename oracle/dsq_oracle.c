/*
 * dsq_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, CPU-only statement of what a DSQ-quantized convolution layer
 * computes once the soft quantizer has been hardened by the sign function
 * (paper: Sec. 3.1 uniform quantizer; Sec. 3.2 remark that phi followed by
 * sgn is the piecewise uniform quantizer; Algorithm 1, feed-forward steps
 * 1, 3, 4 and 5).  It exists so that the GPU library can be checked against
 * something that shares no code with it.  Nothing in the product path may
 * call into this file; only tests, the smoke check and the cpu_baseline leg
 * of the benchmark do.
 *
 * Tensor layouts here are the textbook ones: activations NCHW, weights OIHW,
 * outputs N x C_out x Ho x Wo, one code per byte.  No packing, no tiling, no
 * reordering of the sums.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC
 * (fp contraction is switched off so every fp32 operation below is a single
 * IEEE-754 binary32 operation rounded to nearest-even).
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_BAD_ARG 1
#define ORACLE_NO_MEM 2

int dsq_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int bounds_ok(float l, float u, int bits)
{
    return bits >= 1 && bits <= 8 && isfinite(l) && isfinite(u) && l < u;
}

/* Interval length Delta = (u - l) / (2^b - 1)  (Sec. 3.1, text after the
 * uniform quantizer), evaluated in binary32. */
float dsq_oracle_delta(float l, float u, int bits)
{
    float levels_minus_1 = (float)((1 << bits) - 1);
    float range = u - l;
    return range / levels_minus_1;
}

/* One value -> its code in {0 .. 2^b - 1}.
 *
 * Algorithm 1 step 1 clips to [l, u]; the uniform quantizer of Sec. 3.1
 * rounds the clipped value to the nearest of the 2^b points l + c*Delta.
 * A value exactly half way between two points goes to the upper one: that is
 * what step 3 (sgn of phi, with sgn(0) = +1 from the binary quantizer of
 * Sec. 3.1) yields at x = m_i.  Every operation is binary32, the division is
 * a true division.  A NaN of either kind clips to l: the clip is written as two
 * comparisons (a NaN compares false), not as fmaxf/fminf, whose result for a
 * signalling NaN depends on the C library. */
static int code_of(float x, float l, float u, float delta, int top)
{
    float v = x > l ? x : l;
    v = v < u ? v : u;
    float t = (v - l) / delta;
    float r = floorf(t + 0.5f);
    int c = (int)r;
    if (c < 0) c = 0;
    if (c > top) c = top;
    return c;
}

int dsq_oracle_quantize(const float *x, size_t n, float l, float u, int bits,
                        uint8_t *code)
{
    if (!x || !code || !bounds_ok(l, u, bits)) return ORACLE_BAD_ARG;
    float delta = dsq_oracle_delta(l, u, bits);
    int top = (1 << bits) - 1;
    for (size_t i = 0; i < n; ++i)
        code[i] = (uint8_t)code_of(x[i], l, u, delta, top);
    return ORACLE_OK;
}

/* Weights: the same quantizer with one (l_w, u_w) pair per output channel
 * (Algorithm 1 lists l_w, u_w as layer parameters; a per-tensor pair is the
 * case where all entries are equal).  w is OIHW, per_ch = C_in*R*S. */
int dsq_oracle_quantize_weights(const float *w, const float *lw,
                                const float *uw, int c_out, size_t per_ch,
                                int bits, uint8_t *code)
{
    if (!w || !lw || !uw || !code || c_out <= 0) return ORACLE_BAD_ARG;
    for (int o = 0; o < c_out; ++o) {
        if (!bounds_ok(lw[o], uw[o], bits)) return ORACLE_BAD_ARG;
        int rc = dsq_oracle_quantize(w + (size_t)o * per_ch, per_ch, lw[o],
                                     uw[o], bits, code + (size_t)o * per_ch);
        if (rc) return rc;
    }
    return ORACLE_OK;
}

/* Between two quantized layers of a deployed network the convolution output o
 * of Algorithm 1 step 5 passes through the per-channel affine map a folded
 * batch normalisation leaves behind and, optionally, a ReLU, and is then the
 * input a of the next layer's Algorithm 1.  In binary32, one rounding per
 * operation, multiplication first:
 *     z = y * scale[c];  z = z + shift[c];  z = max(z, 0) if relu
 * y is N x C x (HW), channel-major inside one image. */
int dsq_oracle_affine_relu(const float *y, int n_img, int channels, size_t hw,
                           const float *scale, const float *shift, int relu,
                           float *z)
{
    if (!y || !z || !scale || !shift || n_img <= 0 || channels <= 0) return ORACLE_BAD_ARG;
    for (int n = 0; n < n_img; ++n)
        for (int c = 0; c < channels; ++c) {
            const float *src = y + ((size_t)n * channels + c) * hw;
            float *dst = z + ((size_t)n * channels + c) * hw;
            for (size_t i = 0; i < hw; ++i) {
                float prod = src[i] * scale[c];
                float v = prod + shift[c];
                if (relu) v = fmaxf(v, 0.0f);
                dst[i] = v;
            }
        }
    return ORACLE_OK;
}

/* Algorithm 1 step 4: value = l + Delta * code, as a real number.  l and
 * Delta are the binary32 numbers; the product and sum are done in double,
 * where they are exact (24-bit x 8-bit + 24-bit significands). */
static double level_value(float l, float delta, int c)
{
    return (double)l + (double)delta * (double)c;
}

int dsq_oracle_dequantize(const uint8_t *code, size_t n, float l, float u,
                          int bits, double *value)
{
    if (!code || !value || !bounds_ok(l, u, bits)) return ORACLE_BAD_ARG;
    float delta = dsq_oracle_delta(l, u, bits);
    for (size_t i = 0; i < n; ++i) value[i] = level_value(l, delta, code[i]);
    return ORACLE_OK;
}

typedef struct {
    int N, C_in, H, W, C_out, R, S, stride, pad;
} oracle_geom;

static int geom_ok(const oracle_geom *g)
{
    if (g->N <= 0 || g->C_in <= 0 || g->H <= 0 || g->W <= 0 || g->C_out <= 0 ||
        g->R <= 0 || g->S <= 0 || g->stride <= 0 || g->pad < 0)
        return 0;
    if (g->H + 2 * g->pad < g->R || g->W + 2 * g->pad < g->S) return 0;
    return 1;
}
static int out_h(const oracle_geom *g) { return (g->H + 2 * g->pad - g->R) / g->stride + 1; }
static int out_w(const oracle_geom *g) { return (g->W + 2 * g->pad - g->S) / g->stride + 1; }

/* Integer cross-correlation of the codes themselves.  Taps that fall in the
 * zero padding are left out of the sum.  This is the quantity an integer
 * kernel accumulates before any dequantization. */
static int32_t acc_at(const oracle_geom *g, const uint8_t *a, const uint8_t *w,
                      int n, int o, int oy, int ox)
{
    int32_t acc = 0;
    for (int c = 0; c < g->C_in; ++c)
        for (int r = 0; r < g->R; ++r)
            for (int s = 0; s < g->S; ++s) {
                int iy = oy * g->stride - g->pad + r;
                int ix = ox * g->stride - g->pad + s;
                if (iy < 0 || iy >= g->H || ix < 0 || ix >= g->W) continue;
                int32_t ca = a[(((size_t)n * g->C_in + c) * g->H + iy) * g->W + ix];
                int32_t cw = w[(((size_t)o * g->C_in + c) * g->R + r) * g->S + s];
                acc += ca * cw;
            }
    return acc;
}

int dsq_oracle_conv_codes(const uint8_t *a, const uint8_t *w, int N, int C_in,
                          int H, int W, int C_out, int R, int S, int stride,
                          int pad, int32_t *acc)
{
    oracle_geom g = {N, C_in, H, W, C_out, R, S, stride, pad};
    if (!a || !w || !acc || !geom_ok(&g)) return ORACLE_BAD_ARG;
    int Ho = out_h(&g), Wo = out_w(&g);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int o = 0; o < C_out; ++o)
            for (int oy = 0; oy < Ho; ++oy)
                for (int ox = 0; ox < Wo; ++ox)
                    acc[(((size_t)n * C_out + o) * Ho + oy) * Wo + ox] =
                        acc_at(&g, a, w, n, o, oy, ox);
    return ORACLE_OK;
}

/* Algorithm 1 step 5: o = Convolution(w_hat, a_hat) -- the cross-correlation
 * a deep-learning framework calls convolution (no kernel flip, no bias), zero
 * padding of a_hat (the padded positions hold the real number 0, not the
 * level l_a), summed in double in the order (c, r, s) and rounded once to
 * binary32.  a_hat and w_hat are the dequantized tensors, in double. */
static double real_at(const oracle_geom *g, const double *ahat,
                      const double *what, int n, int o, int oy, int ox)
{
    double sum = 0.0;
    for (int c = 0; c < g->C_in; ++c)
        for (int r = 0; r < g->R; ++r)
            for (int s = 0; s < g->S; ++s) {
                int iy = oy * g->stride - g->pad + r;
                int ix = ox * g->stride - g->pad + s;
                if (iy < 0 || iy >= g->H || ix < 0 || ix >= g->W) continue;
                double av = ahat[(((size_t)n * g->C_in + c) * g->H + iy) * g->W + ix];
                double wv = what[(((size_t)o * g->C_in + c) * g->R + r) * g->S + s];
                sum += av * wv;
            }
    return sum;
}

int dsq_oracle_conv_dequantized(const double *ahat, const double *what, int N,
                                int C_in, int H, int W, int C_out, int R, int S,
                                int stride, int pad, float *out)
{
    oracle_geom g = {N, C_in, H, W, C_out, R, S, stride, pad};
    if (!ahat || !what || !out || !geom_ok(&g)) return ORACLE_BAD_ARG;
    int Ho = out_h(&g), Wo = out_w(&g);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int o = 0; o < C_out; ++o)
            for (int oy = 0; oy < Ho; ++oy)
                for (int ox = 0; ox < Wo; ++ox)
                    out[(((size_t)n * C_out + o) * Ho + oy) * Wo + ox] =
                        (float)real_at(&g, ahat, what, n, o, oy, ox);
    return ORACLE_OK;
}

/* The whole layer from codes: dequantize both tensors (step 4), then step 5. */
int dsq_oracle_conv_real(const uint8_t *a, float la, float ua, const uint8_t *w,
                         const float *lw, const float *uw, int bits, int N,
                         int C_in, int H, int W, int C_out, int R, int S,
                         int stride, int pad, float *out)
{
    oracle_geom g = {N, C_in, H, W, C_out, R, S, stride, pad};
    if (!a || !w || !lw || !uw || !out || !geom_ok(&g)) return ORACLE_BAD_ARG;
    size_t na = (size_t)N * C_in * H * W;
    size_t per_ch = (size_t)C_in * R * S;
    double *ahat = (double *)malloc(na * sizeof(double));
    double *what = (double *)malloc(per_ch * C_out * sizeof(double));
    int rc = ORACLE_NO_MEM;
    if (ahat && what) {
        rc = dsq_oracle_dequantize(a, na, la, ua, bits, ahat);
        for (int o = 0; o < C_out && rc == ORACLE_OK; ++o)
            rc = dsq_oracle_dequantize(w + (size_t)o * per_ch, per_ch, lw[o],
                                       uw[o], bits, what + (size_t)o * per_ch);
        if (rc == ORACLE_OK)
            rc = dsq_oracle_conv_dequantized(ahat, what, N, C_in, H, W, C_out, R,
                                             S, stride, pad, out);
    }
    free(ahat);
    free(what);
    return rc;
}

/* Single outputs of a large layer, one by one: idx[k] is a flat index into
 * the N x C_out x Ho x Wo output.  Levels are formed on the fly with the same
 * step-4 formula, so tensors too large to dequantize whole can be sampled.
 * Either result pointer may be NULL. */
int dsq_oracle_conv_at(const uint8_t *a, float la, float ua, const uint8_t *w,
                       const float *lw, const float *uw, int bits, int N,
                       int C_in, int H, int W, int C_out, int R, int S,
                       int stride, int pad, const int64_t *idx, size_t nidx,
                       float *out_vals, int32_t *acc_vals)
{
    oracle_geom g = {N, C_in, H, W, C_out, R, S, stride, pad};
    if (!a || !w || !lw || !uw || !idx || !geom_ok(&g) || !bounds_ok(la, ua, bits))
        return ORACLE_BAD_ARG;
    int Ho = out_h(&g), Wo = out_w(&g);
    int64_t total = (int64_t)N * C_out * Ho * Wo;
    float da = dsq_oracle_delta(la, ua, bits);
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 16)
    for (size_t k = 0; k < nidx; ++k) {
        int64_t f = idx[k];
        if (f < 0 || f >= total) {
#pragma omp atomic write
            bad = 1;
            continue;
        }
        int ox = (int)(f % Wo); f /= Wo;
        int oy = (int)(f % Ho); f /= Ho;
        int o = (int)(f % C_out);
        int n = (int)(f / C_out);
        if (!bounds_ok(lw[o], uw[o], bits)) {
#pragma omp atomic write
            bad = 1;
            continue;
        }
        float dw = dsq_oracle_delta(lw[o], uw[o], bits);
        if (acc_vals) acc_vals[k] = acc_at(&g, a, w, n, o, oy, ox);
        if (out_vals) {
            double sum = 0.0;
            for (int c = 0; c < C_in; ++c)
                for (int r = 0; r < R; ++r)
                    for (int s = 0; s < S; ++s) {
                        int iy = oy * stride - pad + r;
                        int ix = ox * stride - pad + s;
                        if (iy < 0 || iy >= H || ix < 0 || ix >= W) continue;
                        int ca = a[(((size_t)n * C_in + c) * H + iy) * W + ix];
                        int cw = w[(((size_t)o * C_in + c) * R + r) * S + s];
                        sum += level_value(la, da, ca) * level_value(lw[o], dw, cw);
                    }
            out_vals[k] = (float)sum;
        }
    }
    return bad ? ORACLE_BAD_ARG : ORACLE_OK;
}

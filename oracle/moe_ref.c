/*
 * Reference fused mixture-of-experts feed-forward in fp64 -- TEST INFRASTRUCTURE, not the product.
 *
 * The checker the HIP MoE path is compared against: one thread, plain loops, no blocking, no
 * SIMD intrinsics, no code shared with the GPU path.  Only tests, the smoke check and the
 * bench's cpu_baseline leg may call it.
 *
 * What it computes is the paper's fused-MoE workload (Evaluation, "Kernel Performance": the block-quantized
 * FP8 configuration of DeepSeek-V3.2, model dimension H, intermediate dimension I, top-k routing, the experts of
 * one GPU under expert parallelism; same subsection, "Fused MoE" paragraph: blockwise quantization is
 * preserved, tokens are routed through expert maps, the up-projection intermediates are
 * quantized to FP8 before the down projection).  The paper gives no formulas; the steps below
 * are the published block-quantized recipe that configuration names, written out:
 *
 *   1. activation quantization, per token and per group of 128 consecutive features:
 *        amax = max |x|,  scale = amax * (1/448) (or 1 if amax = 0),  code = e4m3(x * (1/scale))
 *      in fp32 exactly as written (each operation rounded to fp32, 1/scale a true division,
 *      the product clamped to +-448 before rounding to nearest even): a quantised code is a
 *      decision, and both sides must take it in the same precision.
 *   2. for every routed (token t, slot k) whose expert e = ids[t][k] is local (0 <= e < E):
 *        g_j = sum over 128-blocks b of  xs[t][b] * s13[e][j/128][b]       * sum_{h in b} xq[t][h] w13[e][j][h]
 *        u_j = same with row I + j of w13 (gate rows first, then up rows)
 *        a_j = silu(g_j) * u_j,   silu(z) = z / (1 + exp(-z))                       j < I
 *   3. the intermediate a is quantized like step 1 (groups of 128 along j; a rounded to fp32
 *      first), giving aq, as;
 *   4.   o_c = sum over blocks b of  as[b] * s2[e][c/128][b] * sum_{j in b} aq[j] w2[e][c][j]      c < H
 *   5.   y[t][c] = sum over slots k in ascending order of  wts[t][k] * o_c(k)
 *      (slots whose expert is not local contribute nothing: they belong to another GPU).
 *
 * Everything except the quantization decisions of steps 1 and 3 is fp64 on exactly widened
 * inputs.  FP8 is OCP e4m3 (bias 7, 3 mantissa bits, no infinities, 0x7f/0xff NaN, max 448).
 *
 * Layouts (contiguous, row-major): x [T,H] bf16 bits; ids [T,KTOP] int32; wts [T,KTOP] fp32;
 * w13 [E,2I,H] e4m3 bytes; s13 [E,2I/128,H/128] fp32; w2 [E,H,I] e4m3 bytes; s2 [E,H/128,I/128]
 * fp32; y [R,H] fp64 for the R requested tokens.  H and I are multiples of 128.
 * Pinned by tests/test_moe_oracle_pins.py.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static float bf16_bits_to_f32(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* value of an e4m3 code; NaN codes (0x7f, 0xff) decode to NaN */
double moe_ref_e4m3_decode(uint8_t c)
{
    const int sign = c >> 7, e = (c >> 3) & 15, m = c & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexp((double)m, -9);                 /* subnormal: m * 2^-3 * 2^-6 */
    else v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

/* fp32 -> e4m3: clamp to +-448, round to nearest, ties to even.  Finite inputs only. */
uint8_t moe_ref_e4m3_encode(float f)
{
    const uint8_t sign = f < 0.0f || (f == 0.0f && signbit(f)) ? 0x80 : 0x00;
    double a = fabs((double)f);
    if (a >= 448.0) return sign | 0x7e;                   /* 1.75 * 2^8 */
    if (a == 0.0) return sign;
    int ex;
    (void)frexp(a, &ex);                                  /* a = frac * 2^ex, frac in [0.5, 1) */
    int e = ex - 1;                                       /* a in [2^e, 2^(e+1)) */
    if (e < -6) e = -6;                                   /* subnormal range shares the exponent of the smallest normal */
    const double q = ldexp(a, 3 - e);                     /* in units of the spacing 2^(e-3) */
    double r = floor(q);
    const double frac = q - r;
    if (frac > 0.5 || (frac == 0.5 && fmod(r, 2.0) == 1.0)) r += 1.0;
    /* r in [0, 16]: 16 means the next binade */
    int mant = (int)r, be = e + 7;
    if (e == -6 && mant < 8) return sign | (uint8_t)mant; /* subnormal (or zero) */
    if (mant == 16) { mant = 8; be += 1; }
    return sign | (uint8_t)((be << 3) | (mant - 8));
}

/* step 1 / step 3 on one group of 128 fp32 values */
void moe_ref_quant_group(const float *v, uint8_t *code, float *scale)
{
    float amax = 0.0f;
    for (int i = 0; i < 128; ++i) { const float a = fabsf(v[i]); if (a > amax) amax = a; }
    volatile float s = amax * (1.0f / 448.0f);
    if (amax == 0.0f) s = 1.0f;
    volatile float inv = 1.0f / s;
    for (int i = 0; i < 128; ++i) {
        volatile float p = v[i] * inv;
        float c = p;
        if (c > 448.0f) c = 448.0f;
        if (c < -448.0f) c = -448.0f;
        code[i] = moe_ref_e4m3_encode(c);
    }
    *scale = s;
}

/* steps 1-2 for one (token, local expert): a_j in fp64, before it is rounded to fp32 for step 3 */
static void slot_intermediate(const uint16_t *xrow, const uint8_t *w13e, const float *s13e, const double *dec,
                              int H, int I, uint8_t *xq, float *xs, float *xf, double *a)
{
    const int HB = H / 128;
    for (int h = 0; h < H; ++h) xf[h] = bf16_bits_to_f32(xrow[h]);
    for (int b = 0; b < HB; ++b) moe_ref_quant_group(xf + 128 * b, xq + 128 * b, xs + b);
    for (int j = 0; j < I; ++j) {
        double gu[2];
        for (int part = 0; part < 2; ++part) {
            const int row = part * I + j;
            double acc = 0.0;
            for (int b = 0; b < HB; ++b) {
                double blk = 0.0;
                for (int h = 128 * b; h < 128 * b + 128; ++h) blk += dec[xq[h]] * dec[w13e[(size_t)row * (size_t)H + (size_t)h]];
                acc += blk * (double)xs[b] * (double)s13e[(size_t)(row / 128) * (size_t)HB + (size_t)b];
            }
            gu[part] = acc;
        }
        a[j] = gu[0] / (1.0 + exp(-gu[0])) * gu[1];
    }
}

/* step 4 for one row of intermediate codes and scales */
static void slot_down(const uint8_t *aq, const float *as, const uint8_t *w2e, const float *s2e, const double *dec,
                      int H, int I, double *o)
{
    const int IB = I / 128;
    for (int c = 0; c < H; ++c) {
        double acc = 0.0;
        for (int b = 0; b < IB; ++b) {
            double blk = 0.0;
            for (int j = 128 * b; j < 128 * b + 128; ++j) blk += dec[aq[j]] * dec[w2e[(size_t)c * (size_t)I + (size_t)j]];
            acc += blk * (double)as[b] * (double)s2e[(size_t)(c / 128) * (size_t)IB + (size_t)b];
        }
        o[c] = acc;
    }
}

/* The intermediate a [I] (fp64, unrounded) of token t on local expert e.  Returns 0, or nonzero on bad arguments. */
int moe_ref_intermediate_f64(const uint16_t *x, const uint8_t *w13, const float *s13, double *a,
                             int T, int H, int I, int E, int t, int e)
{
    if (!x || !w13 || !s13 || !a || T <= 0 || H <= 0 || I <= 0 || H % 128 || I % 128 || t < 0 || t >= T || e < 0 || e >= E) return 1;
    double dec[256];
    for (int c = 0; c < 256; ++c) dec[c] = moe_ref_e4m3_decode((uint8_t)c);
    uint8_t *xq = malloc((size_t)H);
    float *xs = malloc(sizeof(float) * (size_t)(H / 128)), *xf = malloc(sizeof(float) * (size_t)H);
    if (!xq || !xs || !xf) return 2;
    slot_intermediate(x + (size_t)t * (size_t)H, w13 + (size_t)e * 2 * (size_t)I * (size_t)H,
                      s13 + (size_t)e * 2 * (size_t)(I / 128) * (size_t)(H / 128), dec, H, I, xq, xs, xf, a);
    free(xq); free(xs); free(xf);
    return 0;
}

/* Step 4 alone: o [H] (fp64) from given intermediate codes aq [I] and scales as [I/128] on expert e. */
int moe_ref_down_f64(const uint8_t *aq, const float *as, const uint8_t *w2, const float *s2, double *o,
                     int H, int I, int E, int e)
{
    if (!aq || !as || !w2 || !s2 || !o || H <= 0 || I <= 0 || H % 128 || I % 128 || e < 0 || e >= E) return 1;
    double dec[256];
    for (int c = 0; c < 256; ++c) dec[c] = moe_ref_e4m3_decode((uint8_t)c);
    slot_down(aq, as, w2 + (size_t)e * (size_t)H * (size_t)I, s2 + (size_t)e * (size_t)(H / 128) * (size_t)(I / 128), dec, H, I, o);
    return 0;
}

int moe_ref_f64(const uint16_t *x, const int32_t *ids, const float *wts,
                const uint8_t *w13, const float *s13, const uint8_t *w2, const float *s2,
                double *y, int T, int H, int I, int E, int KTOP, const int *rows, int nrows)
{
    if (!x || !ids || !wts || !w13 || !s13 || !w2 || !s2 || !y) return 1;
    if (T <= 0 || H <= 0 || I <= 0 || E <= 0 || KTOP <= 0 || H % 128 || I % 128) return 1;
    const int R = rows ? nrows : T, HB = H / 128, IB = I / 128;
    double dec[256];
    for (int c = 0; c < 256; ++c) dec[c] = moe_ref_e4m3_decode((uint8_t)c);
    uint8_t *xq = malloc((size_t)H), *aq = malloc((size_t)I);
    float *xs = malloc(sizeof(float) * (size_t)HB), *as = malloc(sizeof(float) * (size_t)IB);
    float *xf = malloc(sizeof(float) * (size_t)H), *af = malloc(sizeof(float) * (size_t)I);
    double *ad = malloc(sizeof(double) * (size_t)I), *od = malloc(sizeof(double) * (size_t)H);
    if (!xq || !aq || !xs || !as || !xf || !af || !ad || !od) return 2;
    for (int r = 0; r < R; ++r) {
        const int t = rows ? rows[r] : r;
        if (t < 0 || t >= T) return 1;
        double *yr = y + (size_t)r * (size_t)H;
        for (int c = 0; c < H; ++c) yr[c] = 0.0;
        for (int k = 0; k < KTOP; ++k) {
            const int e = ids[(size_t)t * (size_t)KTOP + (size_t)k];
            if (e < 0 || e >= E) continue;
            slot_intermediate(x + (size_t)t * (size_t)H, w13 + (size_t)e * 2 * (size_t)I * (size_t)H,
                              s13 + (size_t)e * 2 * (size_t)IB * (size_t)HB, dec, H, I, xq, xs, xf, ad);
            for (int j = 0; j < I; ++j) af[j] = (float)ad[j];
            for (int b = 0; b < IB; ++b) moe_ref_quant_group(af + 128 * b, aq + 128 * b, as + b);
            slot_down(aq, as, w2 + (size_t)e * (size_t)H * (size_t)I, s2 + (size_t)e * (size_t)HB * (size_t)IB, dec, H, I, od);
            const double wk = (double)wts[(size_t)t * (size_t)KTOP + (size_t)k];
            for (int c = 0; c < H; ++c) yr[c] += wk * od[c];
        }
    }
    free(xq); free(aq); free(xs); free(as); free(xf); free(af); free(ad); free(od);
    return 0;
}

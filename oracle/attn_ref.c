/*
 * Reference attention forward in fp64 -- TEST INFRASTRUCTURE, not the product.
 *
 * This file is the checker that the HIP kernels are compared against.  It is
 * deliberately plain: one thread, no tiling, no online softmax, no SIMD
 * intrinsics, no BLAS, and it shares no code with the GPU path.  Only tests,
 * the smoke check and the bench's cpu_baseline leg may call it.
 *
 * What it computes is the textbook definition the paper starts from
 * (the attention definition in its "Motivating Example" section): S = Q K^T, P = softmax(S)
 * row-wise, O = P V.  Flash attention is an exact reorganisation of that
 * definition (tiling + online softmax change only the order of the sums), so
 * the definition itself is the oracle.  Extensions the paper's workload and the
 * library boundary add:
 *   - a scalar multiplier on the scores before the softmax (the paper's
 *     definition has none; callers pass 1/sqrt(D));
 *   - grouped-query attention with contiguous groups, kv head = q head / gqa
 *     (Figure 1: tags of Q use h_q/gqa, K/V tiles are indexed idx_h/gqa);
 *   - the causal mask of the evaluated workload (Evaluation, "Kernel Performance": causal grouped-query attention),
 *     aligned bottom-right: key j is visible to query i iff j <= i + (Sk-Sq);
 *   - the natural-log log-sum-exp of the scaled, visible scores per query row
 *     (not in the paper's kernel; required by the library boundary);
 *   - a query row with no visible key (only possible when Sq > Sk under the
 *     causal mask) yields O = 0 and LSE = -inf.
 *
 * Inputs are bf16 bit patterns (Figure 1 declares Q, K, V, O as bf16); they are
 * widened exactly to fp64 and every operation after that is fp64.
 *
 * Layout: q [B,Hq,Sq,D], k and v [B,Hkv,Sk,D], contiguous, row-major.
 * Pinned by tests/test_oracle_pins.py (closed forms, brute force, invariants).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* exact widening of a bf16 bit pattern: bf16 is the top half of an IEEE fp32 */
static double bf16_bits_to_f64(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/*
 * One query row against one kv head, on fp64 data.
 *   qrow [D]; K, V [Sk, D]; nvis = number of visible keys (keys 0..nvis-1).
 *   scores: caller-provided work array of Sk doubles.
 * Writes orow [D], *lse, and, if probs != NULL, probs[0..Sk-1] (zeros beyond nvis).
 */
static void attn_row_f64(const double *qrow, const double *K, const double *V,
                         int Sk, int D, int nvis, double scale,
                         double *scores, double *orow, double *lse, double *probs)
{
    int j, d;
    if (probs) for (j = 0; j < Sk; ++j) probs[j] = 0.0;
    if (nvis <= 0) {
        for (d = 0; d < D; ++d) orow[d] = 0.0;
        *lse = -INFINITY;
        return;
    }
    /* S = scale * q . k_j */
    for (j = 0; j < nvis; ++j) {
        const double *kr = K + (size_t)j * D;
        double acc = 0.0;
        for (d = 0; d < D; ++d) acc += qrow[d] * kr[d];
        scores[j] = scale * acc;
    }
    /* softmax over the visible keys, max-subtracted */
    double m = scores[0];
    for (j = 1; j < nvis; ++j) if (scores[j] > m) m = scores[j];
    double l = 0.0;
    for (j = 0; j < nvis; ++j) { scores[j] = exp(scores[j] - m); l += scores[j]; }
    *lse = m + log(l);
    /* O = P V */
    for (d = 0; d < D; ++d) orow[d] = 0.0;
    for (j = 0; j < nvis; ++j) {
        const double p = scores[j] / l;
        const double *vr = V + (size_t)j * D;
        if (probs) probs[j] = p;
        for (d = 0; d < D; ++d) orow[d] += p * vr[d];
    }
}

static int visible_keys(int i, int Sq, int Sk, int causal)
{
    if (!causal) return Sk;
    long n = (long)i + (long)(Sk - Sq) + 1; /* keys 0 .. i + (Sk-Sq) */
    if (n < 0) n = 0;
    if (n > Sk) n = Sk;
    return (int)n;
}

static int check_dims(int B, int Hq, int Hkv, int Sq, int Sk, int D)
{
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || Sq <= 0 || Sk <= 0 || D <= 0) return -1;
    if (Hq % Hkv != 0) return -1;
    return 0;
}

/*
 * fp64-input core.  rows == NULL: every query row, o is [B,Hq,Sq,D], lse [B,Hq,Sq].
 * rows != NULL: rows is [B*Hq, nrows] (query indices chosen per (b,h)),
 * o is [B,Hq,nrows,D], lse [B,Hq,nrows].
 * Returns 0, or -1 on bad dimensions / row index, -2 on allocation failure.
 */
int attn_ref_f64_from_f64(const double *q, const double *k, const double *v,
                          double *o, double *lse,
                          int B, int Hq, int Hkv, int Sq, int Sk, int D,
                          int causal, double scale, const int *rows, int nrows)
{
    if (check_dims(B, Hq, Hkv, Sq, Sk, D)) return -1;
    if (rows && nrows <= 0) return -1;
    const int gqa = Hq / Hkv;
    const int R = rows ? nrows : Sq;
    double *scores = (double *)malloc(sizeof(double) * (size_t)Sk);
    if (!scores) return -2;
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hq; ++h) {
            const int hk = h / gqa;
            const double *Kh = k + ((size_t)b * Hkv + hk) * (size_t)Sk * D;
            const double *Vh = v + ((size_t)b * Hkv + hk) * (size_t)Sk * D;
            const size_t bh = (size_t)b * Hq + h;
            for (int r = 0; r < R; ++r) {
                const int i = rows ? rows[bh * (size_t)nrows + r] : r;
                if (i < 0 || i >= Sq) { free(scores); return -1; }
                const double *qrow = q + (bh * (size_t)Sq + i) * (size_t)D;
                attn_row_f64(qrow, Kh, Vh, Sk, D, visible_keys(i, Sq, Sk, causal), scale,
                             scores, o + (bh * (size_t)R + r) * (size_t)D, lse + bh * (size_t)R + r, NULL);
            }
        }
    free(scores);
    return 0;
}

/*
 * bf16-input entry point (the one the parity tests use).  Same conventions as
 * above; q, k, v hold bf16 bit patterns.  K and V of one kv head are widened to
 * fp64 once and reused by the gqa query heads that read it.
 */
int attn_ref_f64(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                 double *o, double *lse,
                 int B, int Hq, int Hkv, int Sq, int Sk, int D,
                 int causal, double scale, const int *rows, int nrows)
{
    if (check_dims(B, Hq, Hkv, Sq, Sk, D)) return -1;
    if (rows && nrows <= 0) return -1;
    const int gqa = Hq / Hkv;
    const int R = rows ? nrows : Sq;
    const size_t slab = (size_t)Sk * D;
    double *Kd = (double *)malloc(sizeof(double) * slab);
    double *Vd = (double *)malloc(sizeof(double) * slab);
    double *qd = (double *)malloc(sizeof(double) * (size_t)D);
    double *scores = (double *)malloc(sizeof(double) * (size_t)Sk);
    int rc = 0;
    if (!Kd || !Vd || !qd || !scores) { rc = -2; goto done; }
    for (int b = 0; b < B; ++b)
        for (int hk = 0; hk < Hkv; ++hk) {
            const uint16_t *Kh = k + ((size_t)b * Hkv + hk) * slab;
            const uint16_t *Vh = v + ((size_t)b * Hkv + hk) * slab;
            for (size_t t = 0; t < slab; ++t) { Kd[t] = bf16_bits_to_f64(Kh[t]); Vd[t] = bf16_bits_to_f64(Vh[t]); }
            for (int h = hk * gqa; h < (hk + 1) * gqa; ++h) {
                const size_t bh = (size_t)b * Hq + h;
                for (int r = 0; r < R; ++r) {
                    const int i = rows ? rows[bh * (size_t)nrows + r] : r;
                    if (i < 0 || i >= Sq) { rc = -1; goto done; }
                    const uint16_t *qrow = q + (bh * (size_t)Sq + i) * (size_t)D;
                    for (int d = 0; d < D; ++d) qd[d] = bf16_bits_to_f64(qrow[d]);
                    attn_row_f64(qd, Kd, Vd, Sk, D, visible_keys(i, Sq, Sk, causal), scale,
                                 scores, o + (bh * (size_t)R + r) * (size_t)D, lse + bh * (size_t)R + r, NULL);
                }
            }
        }
done:
    free(Kd); free(Vd); free(qd); free(scores);
    return rc;
}

/*
 * Debug view used by the "softmax rows sum to one" pin: the probabilities of one
 * query row (b, h, i), written to probs[0..Sk-1] (zero for masked keys), plus
 * that row's O [D] and LSE.
 */
int attn_ref_row_probs_f64(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                           int B, int Hq, int Hkv, int Sq, int Sk, int D,
                           int causal, double scale, int b, int h, int i,
                           double *probs, double *orow, double *lse)
{
    if (check_dims(B, Hq, Hkv, Sq, Sk, D)) return -1;
    if (b < 0 || b >= B || h < 0 || h >= Hq || i < 0 || i >= Sq) return -1;
    const int hk = h / (Hq / Hkv);
    const size_t slab = (size_t)Sk * D;
    double *Kd = (double *)malloc(sizeof(double) * slab);
    double *Vd = (double *)malloc(sizeof(double) * slab);
    double *qd = (double *)malloc(sizeof(double) * (size_t)D);
    double *scores = (double *)malloc(sizeof(double) * (size_t)Sk);
    int rc = 0;
    if (!Kd || !Vd || !qd || !scores) { rc = -2; goto done; }
    const uint16_t *Kh = k + ((size_t)b * Hkv + hk) * slab;
    const uint16_t *Vh = v + ((size_t)b * Hkv + hk) * slab;
    for (size_t t = 0; t < slab; ++t) { Kd[t] = bf16_bits_to_f64(Kh[t]); Vd[t] = bf16_bits_to_f64(Vh[t]); }
    const uint16_t *qrow = q + (((size_t)b * Hq + h) * (size_t)Sq + i) * (size_t)D;
    for (int d = 0; d < D; ++d) qd[d] = bf16_bits_to_f64(qrow[d]);
    attn_row_f64(qd, Kd, Vd, Sk, D, visible_keys(i, Sq, Sk, causal), scale, scores, orow, lse, probs);
done:
    free(Kd); free(Vd); free(qd); free(scores);
    return rc;
}

/*
 * Reference bf16 matrix product in fp64 -- TEST INFRASTRUCTURE, not the product.
 *
 * The checker the HIP GEMM kernel is compared against.  Deliberately plain: one
 * thread, three nested loops, no blocking, no SIMD intrinsics, no BLAS, no code
 * shared with the GPU path.  Only tests, the smoke check and the bench's
 * cpu_baseline leg may call it.
 *
 * What it computes is the definition of the paper's GEMM workload (Evaluation,
 * "Kernel Performance": products of square bf16 matrices): C = A B with A [M,K] and B [K,N],
 * c_ij = sum_k a_ik b_kj.  The paper does not say how B lies in memory, so both
 * row-major storages are supported: b_is_nk = 0 reads B as [K,N] (b_kj at
 * b[k*ldb + j]); b_is_nk = 1 reads it as [N,K] (b_kj at b[j*ldb + k]), the layout
 * of a linear layer's weight, C = A W^T.  Inputs are bf16 bit patterns widened
 * exactly to fp64; every operation after that is fp64; no output rounding.
 *
 * Next to each c_ij the absolute sum  s_ij = sum_k |a_ik| |b_kj|  can be returned:
 * the parity tests scale their floating-point tolerance by it.
 *
 * Leading dimensions are in elements and may exceed the row length.
 * Pinned by tests/test_gemm_oracle_pins.py.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

static double bf16_bits_to_f64(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static int bad_dims(int M, int N, int K, long long lda, long long ldb, int b_is_nk)
{
    if (M <= 0 || N <= 0 || K <= 0) return 1;
    if (lda < K) return 1;
    if (ldb < (b_is_nk ? K : N)) return 1;
    return 0;
}

/* one output element and its absolute sum */
static void dot_ij(const uint16_t *a, const uint16_t *b, int i, int j, int K,
                   long long lda, long long ldb, int b_is_nk, double *c, double *s)
{
    double acc = 0.0, abs_acc = 0.0;
    for (int k = 0; k < K; ++k) {
        const double x = bf16_bits_to_f64(a[(size_t)i * (size_t)lda + (size_t)k]);
        const double y = b_is_nk ? bf16_bits_to_f64(b[(size_t)j * (size_t)ldb + (size_t)k])
                                 : bf16_bits_to_f64(b[(size_t)k * (size_t)ldb + (size_t)j]);
        acc += x * y;
        abs_acc += fabs(x) * fabs(y);
    }
    *c = acc;
    *s = abs_acc;
}

/* c [M,N] contiguous (fp64); cabs [M,N] contiguous or NULL.  Returns 0, or 1 on bad arguments. */
int gemm_ref_f64(const uint16_t *a, const uint16_t *b, double *c, double *cabs,
                 int M, int N, int K, long long lda, long long ldb, int b_is_nk)
{
    if (!a || !b || !c || bad_dims(M, N, K, lda, ldb, b_is_nk)) return 1;
    for (int i = 0; i < M; ++i)
        for (int j = 0; j < N; ++j) {
            double v, s;
            dot_ij(a, b, i, j, K, lda, ldb, b_is_nk, &v, &s);
            c[(size_t)i * (size_t)N + (size_t)j] = v;
            if (cabs) cabs[(size_t)i * (size_t)N + (size_t)j] = s;
        }
    return 0;
}

/* n sampled outputs: out[t] = c[si[t], sj[t]]; outabs may be NULL.  Returns 0, or 1 on bad arguments. */
int gemm_ref_f64_samples(const uint16_t *a, const uint16_t *b, const int *si, const int *sj, int n,
                         double *out, double *outabs,
                         int M, int N, int K, long long lda, long long ldb, int b_is_nk)
{
    if (!a || !b || !si || !sj || !out || n < 0 || bad_dims(M, N, K, lda, ldb, b_is_nk)) return 1;
    for (int t = 0; t < n; ++t) {
        if (si[t] < 0 || si[t] >= M || sj[t] < 0 || sj[t] >= N) return 1;
        double v, s;
        dot_ij(a, b, si[t], sj[t], K, lda, ldb, b_is_nk, &v, &s);
        out[t] = v;
        if (outabs) outabs[t] = s;
    }
    return 0;
}

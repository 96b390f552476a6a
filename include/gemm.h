/*
 * gemm.h -- C ABI of the MI355X (gfx950) bf16 matrix product.
 *
 * Operation (the GEMM workload of the paper's Evaluation, "Kernel Performance": products of
 * square bf16 matrices whose entries are normal draws; Table 2 lists the optimizations a fast
 * kernel for it combines):
 *
 *     C[i,j] = sum_{k < K} A[i,k] * B[k,j]          i < M, j < N
 *
 * with bf16 inputs, fp32 accumulation on the matrix cores, and one rounding of each
 * C element to bf16 (nearest even) when it is stored.  The paper does not say how B is
 * stored; both row-major storages are accepted:
 *     b_is_nk == 0 :  B is [K, N], element (k,j) at b[k*ldb + j]    (plain C = A B)
 *     b_is_nk != 0 :  B is [N, K], element (k,j) at b[j*ldb + k]    (C = A W^T, a linear
 *                                                                   layer's weight)
 * A is [M, K] row-major with row pitch lda, C is [M, N] row-major with row pitch ldc;
 * pitches are in ELEMENTS and may exceed the row length (sub-matrices of wider arrays).
 *
 * All pointers are DEVICE pointers into caller-owned memory; the library neither
 * allocates nor frees nor synchronises.  c must not overlap a or b.  Inputs must be
 * finite (an Inf or NaN propagates as in the definition).
 *
 * Supported: any M, N, K >= 1 with lda >= K, ldb >= (b_is_nk ? K : N), ldc >= N and every
 * pitch < 2^31.  The tiled matrix-core kernel runs when a, b, c are 16-byte aligned and
 * N, K, lda, ldb, ldc are multiples of 8 (M is free); any other shape runs a slower
 * general kernel with the same result contract.  Pointers must be 2-byte aligned.
 *
 * `stream` is a hipStream_t passed as void* (NULL = the default stream).  The call
 * enqueues one kernel and returns.  Thread-safe, no global state.  Every argument check
 * precedes the first HIP call.  Return codes are those of attn.h (ATTN_OK, ATTN_ERR_*;
 * attn_strerror describes them): NULL_PTR (a, b or c NULL), BAD_SHAPE (a dimension <= 0, a
 * pitch shorter than its row or >= 2^31, more than 2^31-1 tiles), MISALIGNED (odd pointer),
 * LAUNCH (the HIP runtime refused the launch).
 */
#ifndef GEMM_MI355X_H
#define GEMM_MI355X_H

#ifdef __cplusplus
extern "C" {
#endif

int gemm_bf16(const void *a, const void *b, void *c, int M, int N, int K,
              long long lda, long long ldb, long long ldc, int b_is_nk, void *stream);

/*
 * The same product with the workgroup tile of the matrix-core kernel chosen by the caller
 * ("tile-size specialization" in the paper's Table 2): tile = 256 (256 x 256 tiles, one
 * workgroup per CU, two LDS stages 64 deep in k), 2564 (the same tile in four stages 32 deep),
 * 128 (128 x 128 tiles in two stages, two workgroups per CU), 1284 (128 x 128 tiles in four stages,
 * one per CU), 64 (64 x 64 tiles by two wavefronts, four stages): these run v_mfma_f32_32x32x16_bf16.
 * The same five shapes on v_mfma_f32_16x16x32_bf16, which takes less power per FLOP and is faster wherever the
 * power limit sets the clock (large products of normally distributed data): 25616, 256416, 12816, 128416, 6416;
 * and 19216: 192 x 256 tiles (192 rows of C) on that instruction, for results that 256 x 256 tiles cut into a
 * poor number of workgroups (3072 x 3072: 192 instead of 144 for 256 CUs).
 * 0 = what gemm_bf16 does: of 25616, 19216, 128, 1284 and 64 the shape with the best estimate of (throughput of the
 * shape on a full chip) x (how full its last round of workgroups leaves the 256 CUs); see gemm_bf16_auto_tile.
 * Any other value: ATTN_ERR_UNSUPPORTED.  Shapes that only the general kernel can take ignore the choice.
 * For tuning and for tests.
 */
int gemm_bf16_tile(const void *a, const void *b, void *c, int M, int N, int K,
                   long long lda, long long ldb, long long ldc, int b_is_nk, int tile, void *stream);

/* The tile gemm_bf16 takes for an M x N result when its operands qualify for the matrix-core kernel: 64, 128,
 * 1284, 19216 or 25616 as described above (0 for invalid sizes).  Host-only helper, for tuning and for tests. */
int gemm_bf16_auto_tile(int M, int N);

/* Algorithmic FLOPs of one gemm_bf16 call: 2*M*N*K (0 for invalid sizes).  Host-only helper. */
double gemm_bf16_flops(int M, int N, int K);

#ifdef __cplusplus
}
#endif
#endif

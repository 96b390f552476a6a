// C ABI of the bf16 matrix product: argument validation and dispatch.  Every check runs
// before the first HIP call.  See include/gemm.h for the contract.
#include <stdint.h>

#include "../../include/attn.h"
#include "../../include/gemm.h"
#include "gemm_launch.h"

extern "C" int gemm_bf16_tile(const void* a, const void* b, void* c, int M, int N, int K,
                              long long lda, long long ldb, long long ldc, int b_is_nk, int tile, void* stream) {
    if (!a || !b || !c) return ATTN_ERR_NULL_PTR;
    if (tile != 0 && tile != 64 && tile != 128 && tile != 256 && tile != 2564 && tile != 1284 && tile != 25616 && tile != 19216 && tile != 256416 && tile != 12816 && tile != 128416 && tile != 6416) return ATTN_ERR_UNSUPPORTED;
    if (M <= 0 || N <= 0 || K <= 0) return ATTN_ERR_BAD_SHAPE;
    if (lda < K || ldb < (b_is_nk ? K : N) || ldc < N) return ATTN_ERR_BAD_SHAPE;
    if (lda >= (1LL << 31) || ldb >= (1LL << 31) || ldc >= (1LL << 31)) return ATTN_ERR_BAD_SHAPE;
    // the smallest tile any kernel here uses is 64 x 64: bound the grid for all of them
    if ((((long long)M + 63) / 64) * (((long long)N + 63) / 64) >= (1LL << 31)) return ATTN_ERR_BAD_SHAPE;
    if (((uintptr_t)a | (uintptr_t)b | (uintptr_t)c) & 1u) return ATTN_ERR_MISALIGNED;

    // The matrix-core kernel moves 16-byte pieces: every row start and every 8-element
    // piece of a row must be 16-byte aligned, and its per-lane byte offsets inside a
    // 256-row tile are 32-bit.
    const bool aligned = ((((uintptr_t)a | (uintptr_t)b | (uintptr_t)c) & 15u) == 0) &&
                         (((long long)N | (long long)K | lda | ldb | ldc) & 7) == 0;
    const bool small_pitch = lda < (1LL << 22) && ldb < (1LL << 22);

    GemmParams p;
    p.a = (const __bf16*)a; p.b = (const __bf16*)b; p.c = (__bf16*)c;
    p.M = M; p.N = N; p.K = K;
    p.lda = lda; p.ldb = ldb; p.ldc = ldc;
    p.tiles_m = 0; p.tiles_n = 0;
    return gemm_launch(p, b_is_nk != 0, aligned && small_pitch, tile, (hipStream_t)stream) == 0 ? ATTN_OK : ATTN_ERR_LAUNCH;
}

extern "C" int gemm_bf16(const void* a, const void* b, void* c, int M, int N, int K,
                         long long lda, long long ldb, long long ldc, int b_is_nk, void* stream) {
    return gemm_bf16_tile(a, b, c, M, N, K, lda, ldb, ldc, b_is_nk, 0, stream);
}

extern "C" int gemm_bf16_auto_tile(int M, int N) {
    if (M <= 0 || N <= 0) return 0;
    return gemm_auto_tile(M, N);
}

extern "C" double gemm_bf16_flops(int M, int N, int K) {
    if (M <= 0 || N <= 0 || K <= 0) return 0.0;
    return 2.0 * (double)M * (double)N * (double)K;
}

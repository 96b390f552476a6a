// Internal interface between the C-ABI translation unit (argument checks, no device
// code) and the GEMM kernel translation unit.
#pragma once
#include <hip/hip_runtime.h>

struct GemmParams {
    const __bf16* a;   // [M, K], row pitch lda
    const __bf16* b;   // [K, N] (row pitch ldb) or, if b_is_nk, [N, K]
    __bf16* c;         // [M, N], row pitch ldc
    int M, N, K;
    long long lda, ldb, ldc;   // elements
    int tiles_m, tiles_n;      // set by the launcher for the kernel it picks
};

// Enqueue the product on `stream`; `tiled` says whether the operands satisfy the
// alignment rules of the matrix-core kernel; `tile` is 0 (choose by size), 128 or 256.
// Returns 0, or -1 if the launch was refused.
int gemm_launch(GemmParams p, int b_is_nk, bool tiled, int tile, hipStream_t stream);

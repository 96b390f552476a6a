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

// The workgroup tile gemm_launch takes for an M x N result when the caller leaves the choice open
// (64, 128, 1284 or 256: see gemm_bf16_tile in include/gemm.h).  Host arithmetic only.
int gemm_auto_tile(int M, int N);

// Enqueue the product on `stream`; `tiled` says whether the operands satisfy the
// alignment rules of the matrix-core kernel; `tile` is 0 (gemm_auto_tile) or one of the values
// gemm_bf16_tile accepts.  Returns 0, or -1 if the launch was refused.
int gemm_launch(GemmParams p, int b_is_nk, bool tiled, int tile, hipStream_t stream);

// Internal interface between the C-ABI translation unit (argument checks, no device
// code) and the kernel translation unit.
#pragma once
#include <hip/hip_runtime.h>

struct AttnParams {
    const __bf16* q;
    const __bf16* k;
    const __bf16* v;
    __bf16* o;
    float* lse;        // may be null
    int B, Hq, Hkv, Sq, Sk;
    // element strides: batch, head, sequence row (the D elements of a row are contiguous)
    long long q_sb, q_sh, q_ss, k_sb, k_sh, k_ss, v_sb, v_sh, v_ss, o_sb, o_sh, o_ss;
    int nQt;           // query tiles per head (set by the launcher for the kernel it picks)
    int nblocks;       // B * (Hq / hpw) * nQt  (set by the launcher)
    int hpw, hpw_log2; // query heads of one kv head that a workgroup covers side by side: 1, 2, 4 or 8 (set by the launcher)
    float scale;       // multiplier on q.k before the softmax
    float scale_log2;  // scale * log2(e): scores are exponentiated with exp2
};

// Enqueue the forward kernel for head dimension D (64 or 128) on `stream`.  wg_rows: query rows per workgroup
// of the tiled kernel, 256 or 128, or 0 for the launcher's own choice.
// Returns 0, -1 if the runtime refused the launch, -2 if the grid would not fit 31 bits.
int attn_launch(AttnParams p, int D, int causal, int wg_rows, hipStream_t stream);

// Enqueue the pure-MFMA calibration kernel (blocks x 8 wavefronts x iters x 4 MFMAs); returns
// the FLOPs it performs, or -1 if the launch was refused.  sink: >= 4 bytes of device memory.
double attn_launch_mfma_calibration(float* sink, int blocks, int iters, int data, hipStream_t stream);

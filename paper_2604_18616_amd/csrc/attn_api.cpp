// C ABI of the attention-forward library: argument validation and dispatch.
// Every check below runs before the first HIP call, so the error paths work on a
// machine without a GPU.  See include/attn.h for the contract.
#include <math.h>
#include <stdint.h>

#include "../../include/attn.h"
#include "attn_launch.h"

#define ATTN_VERSION 100   /* 0.1.0 */

static int check_dims(int B, int Hq, int Hkv, int Sq, int Sk, int D) {
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || Sq <= 0 || Sk <= 0 || D <= 0) return ATTN_ERR_BAD_SHAPE;
    if (Hq % Hkv != 0) return ATTN_ERR_BAD_SHAPE;
    return ATTN_OK;
}

// Common path of both entry points.  Strides are in elements: {batch, head, row}.
static int attn_fwd_impl(const void* q, const void* k, const void* v, void* o, float* lse,
                         int B, int Hq, int Hkv, int Sq, int Sk, int D,
                         const long long* qs, const long long* ks, const long long* vs, const long long* os,
                         int causal, float scale, int wg_rows, void* stream) {
    if (!q || !k || !v || !o) return ATTN_ERR_NULL_PTR;
    if (wg_rows != 0 && wg_rows != 128 && wg_rows != 256) return ATTN_ERR_UNSUPPORTED;
    if (int rc = check_dims(B, Hq, Hkv, Sq, Sk, D)) return rc;
    if (D != 64 && D != 128) return ATTN_ERR_UNSUPPORTED;
    const long long nQt = ((long long)Sq + 127) / 128;
    const long long nblocks = (long long)B * Hq * nQt;
    if (nblocks >= (1LL << 31)) return ATTN_ERR_BAD_SHAPE;
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o) & 15u) return ATTN_ERR_MISALIGNED;
    if (lse && ((uintptr_t)lse & 3u)) return ATTN_ERR_MISALIGNED;
    const long long* all[4] = {qs, ks, vs, os};
    for (int t = 0; t < 4; ++t) {
        if (all[t][2] < D || all[t][0] < 0 || all[t][1] < 0) return ATTN_ERR_BAD_SHAPE;     // rows may not overlap
        if ((all[t][0] | all[t][1] | all[t][2]) & 7) return ATTN_ERR_MISALIGNED;            // keep every row 16-byte aligned
        if (all[t][2] >= (1LL << 28)) return ATTN_ERR_BAD_SHAPE;
    }
    if (!(scale > 0.0f) || isinf(scale)) return ATTN_ERR_BAD_SCALE;   // rejects NaN, <= 0, inf

    AttnParams p;
    p.q = (const __bf16*)q; p.k = (const __bf16*)k; p.v = (const __bf16*)v;
    p.o = (__bf16*)o; p.lse = lse;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.Sq = Sq; p.Sk = Sk;
    p.q_sb = qs[0]; p.q_sh = qs[1]; p.q_ss = qs[2];
    p.k_sb = ks[0]; p.k_sh = ks[1]; p.k_ss = ks[2];
    p.v_sb = vs[0]; p.v_sh = vs[1]; p.v_ss = vs[2];
    p.o_sb = os[0]; p.o_sh = os[1]; p.o_ss = os[2];
    p.nQt = 0; p.nblocks = 0; p.hpw = 1; p.hpw_log2 = 0;   // set by the launcher
    p.scale = scale;
    p.scale_log2 = (float)((double)scale * 1.4426950408889634074);
    const int rc = attn_launch(p, D, causal != 0, wg_rows, (hipStream_t)stream);
    return rc == 0 ? ATTN_OK : rc == -2 ? ATTN_ERR_BAD_SHAPE : ATTN_ERR_LAUNCH;
}

extern "C" int attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                        int B, int Hq, int Hkv, int Sq, int Sk, int D,
                        int causal, float scale, void* stream) {
    if (int rc = check_dims(B, Hq, Hkv, Sq, Sk, D)) return (q && k && v && o) ? rc : ATTN_ERR_NULL_PTR;
    const long long qs[3] = {(long long)Hq * Sq * D, (long long)Sq * D, D};
    const long long ks[3] = {(long long)Hkv * Sk * D, (long long)Sk * D, D};
    return attn_fwd_impl(q, k, v, o, lse, B, Hq, Hkv, Sq, Sk, D, qs, ks, ks, qs, causal, scale, 0, stream);
}

extern "C" int attn_fwd_strided(const void* q, const void* k, const void* v, void* o, float* lse,
                                int B, int Hq, int Hkv, int Sq, int Sk, int D,
                                const long long* q_strides, const long long* k_strides,
                                const long long* v_strides, const long long* o_strides,
                                int causal, float scale, void* stream) {
    if (!q_strides || !k_strides || !v_strides || !o_strides) return ATTN_ERR_NULL_PTR;
    return attn_fwd_impl(q, k, v, o, lse, B, Hq, Hkv, Sq, Sk, D, q_strides, k_strides, v_strides, o_strides,
                         causal, scale, 0, stream);
}

extern "C" int attn_fwd_tile(const void* q, const void* k, const void* v, void* o, float* lse,
                             int B, int Hq, int Hkv, int Sq, int Sk, int D,
                             int causal, float scale, int wg_rows, void* stream) {
    if (int rc = check_dims(B, Hq, Hkv, Sq, Sk, D)) return (q && k && v && o) ? rc : ATTN_ERR_NULL_PTR;
    const long long qs[3] = {(long long)Hq * Sq * D, (long long)Sq * D, D};
    const long long ks[3] = {(long long)Hkv * Sk * D, (long long)Sk * D, D};
    return attn_fwd_impl(q, k, v, o, lse, B, Hq, Hkv, Sq, Sk, D, qs, ks, ks, qs, causal, scale, wg_rows, stream);
}

extern "C" double attn_mfma_calibration(float* sink, int blocks, int iters, void* stream) {
    if (!sink || blocks <= 0 || iters <= 0) return -1.0;
    return attn_launch_mfma_calibration(sink, blocks, iters, 0, (hipStream_t)stream);
}

extern "C" double attn_mfma_calibration_data(float* sink, int blocks, int iters, int data, void* stream) {
    if (!sink || blocks <= 0 || iters <= 0 || data < 0 || data > 5) return -1.0;
    return attn_launch_mfma_calibration(sink, blocks, iters, data, (hipStream_t)stream);
}

extern "C" int attn_device_info(int device, int* cus, int* clock_khz, double* bf16_peak_tflops) {
    if (device < 0) return ATTN_ERR_BAD_SHAPE;
    int n = 0, c = 0, khz = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || device >= n) return ATTN_ERR_LAUNCH;
    if (hipDeviceGetAttribute(&c, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) return ATTN_ERR_LAUNCH;
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, device) != hipSuccess) return ATTN_ERR_LAUNCH;
    if (cus) *cus = c;
    if (clock_khz) *clock_khz = khz;
    if (bf16_peak_tflops) *bf16_peak_tflops = (double)c * 4096.0 * (double)khz * 1e3 / 1e12;
    return ATTN_OK;
}

extern "C" const char* attn_strerror(int code) {
    switch (code) {
        case ATTN_OK:              return "success";
        case ATTN_ERR_NULL_PTR:    return "q, k, v or o is NULL";
        case ATTN_ERR_BAD_SHAPE:   return "bad shape: a dimension is <= 0, Hq is not a multiple of Hkv, or the grid overflows";
        case ATTN_ERR_UNSUPPORTED: return "unsupported head dimension (D must be 64 or 128)";
        case ATTN_ERR_MISALIGNED:  return "misaligned pointer (q/k/v/o need 16 bytes, lse 4 bytes)";
        case ATTN_ERR_BAD_SCALE:   return "scale must be finite and > 0";
        case ATTN_ERR_LAUNCH:      return "the HIP runtime refused the kernel launch";
        case ATTN_ERR_TOO_LARGE:   return "sizes exceed a fixed capacity of the library (moe_ffn_fp8_static: the workspace these sizes need is larger than the library-owned scratch array)";
        default:                   return "unknown attn error code";
    }
}

extern "C" int attn_version(void) { return ATTN_VERSION; }

extern "C" double attn_fwd_flops(int B, int Hq, int Hkv, int Sq, int Sk, int D, int causal) {
    if (check_dims(B, Hq, Hkv, Sq, Sk, D)) return -1.0;
    double pairs;
    if (!causal) {
        pairs = (double)Sq * (double)Sk;
    } else {
        // row i sees min(Sk, max(0, i + (Sk - Sq) + 1)) keys: an arithmetic series that ends at Sk in row Sq - 1
        // and starts at row i0 = max(0, Sq - Sk) with first = i0 + (Sk - Sq) + 1 keys
        const long long i0 = Sq > Sk ? (long long)Sq - Sk : 0;
        const long long m = (long long)Sq - i0, first = i0 + ((long long)Sk - Sq) + 1;
        pairs = 0.5 * (double)m * (double)(first + Sk);
    }
    return 4.0 * D * (double)B * (double)Hq * pairs;
}

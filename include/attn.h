/*
 * attn.h -- C ABI of the MI355X (gfx950) flash-attention forward library.
 *
 * Operation (the attention definition of the paper's "Motivating Example": S = Q K^T, P = softmax(S)
 * row-wise, O = P V, computed tile by tile with an online softmax so that S is
 * never materialised; Figure 1 gives the tiled kernel this library re-designs
 * for CDNA4):
 *
 *     s_ij   = scale * sum_d Q[b,h,i,d] * K[b,hk,j,d]        hk = h / (Hq/Hkv)
 *     J(i)   = { j in [0,Sk) : !causal  or  j <= i + (Sk - Sq) }
 *     lse_i  = ln sum_{j in J(i)} exp(s_ij)
 *     O[b,h,i,:] = sum_{j in J(i)} exp(s_ij - lse_i) * V[b,hk,j,:]
 *
 * The paper's definition carries no scale; the workload it evaluates is causal
 * grouped-query attention in bf16 with fp32 accumulation (Evaluation, "Kernel Performance"; Figure 1:
 * kv head = q head / gqa).  Scores, running max / sum and the output
 * accumulator are fp32; only P is rounded to bf16 (as the second MFMA operand)
 * and O is rounded once, to nearest even, when stored.
 *
 * All pointers are DEVICE pointers into caller-owned memory; the library
 * neither allocates nor frees nor synchronises.  Tensors are contiguous and
 * row-major:
 *     q   : bf16 [B, Hq,  Sq, D]
 *     k,v : bf16 [B, Hkv, Sk, D]
 *     o   : bf16 [B, Hq,  Sq, D]     (written)
 *     lse : fp32 [B, Hq,  Sq]        (written; may be NULL -> not written)
 * q, k, v, o must be 16-byte aligned, lse 4-byte aligned.  o/lse must not alias
 * the inputs.  A query row with no visible key (causal and Sq > Sk only) gets
 * O = 0 and lse = -inf.
 *
 * Supported: D in {64, 128}; any B, Hq, Hkv, Sq, Sk >= 1 with Hq % Hkv == 0 and
 * B*Hq*ceil(Sq/128) < 2^31; scale finite and > 0.
 *
 * `stream` is a hipStream_t passed as void* (NULL = the default stream).  The
 * call enqueues the kernel on that stream and returns; the result is ready
 * when the stream reaches that point.  Thread-safe, no global state.
 *
 * Every argument check happens before the first HIP call, so error paths can be
 * exercised on a machine without a GPU.  Nothing is ever silently wrong: an
 * unsupported request returns an error and launches nothing.
 */
#ifndef ATTN_MI355X_H
#define ATTN_MI355X_H

#ifdef __cplusplus
extern "C" {
#endif

enum {
    ATTN_OK              =  0,
    ATTN_ERR_NULL_PTR    = -1,  /* q, k, v or o is NULL                               */
    ATTN_ERR_BAD_SHAPE   = -2,  /* a dimension <= 0, Hq % Hkv != 0, or grid overflow  */
    ATTN_ERR_UNSUPPORTED = -3,  /* D not in {64,128}                                  */
    ATTN_ERR_MISALIGNED  = -4,  /* q/k/v/o not 16-byte aligned, lse not 4-byte aligned */
    ATTN_ERR_BAD_SCALE   = -5,  /* scale is NaN, infinite, zero or negative           */
    ATTN_ERR_LAUNCH      = -6,  /* the HIP runtime refused the launch                 */
    ATTN_ERR_TOO_LARGE   = -7   /* sizes exceed a fixed capacity of the library (moe.h: the library-owned scratch) */
};

/*
 * Flash-attention forward ("Motivating Example" definition; Figure 1 tiling; Evaluation's
 * causal GQA workload).  Returns ATTN_OK or a negative ATTN_ERR_* code.
 * causal: 0 = all keys visible, non-zero = bottom-right aligned causal mask.
 */
int attn_fwd(const void *q, const void *k, const void *v, void *o, float *lse,
             int B, int Hq, int Hkv, int Sq, int Sk, int D,
             int causal, float scale, void *stream);

/*
 * The same operation on tensors with arbitrary batch / head / row strides (the paper's own
 * kernel, Figure 1, takes Q, K, V, O as [seq, head, d]; a [B, S, H, D] buffer is
 * strides {S*H*D, D, H*D}).  Each *_strides points to 3 HOST integers {batch, head, row}
 * in ELEMENTS; the D elements of a row are contiguous.  Every stride must be a multiple of
 * 8 elements (rows stay 16-byte aligned), row stride >= D and < 2^28, none negative; o must
 * not overlap itself or the inputs.  lse is always contiguous [B, Hq, Sq].  Everything else
 * (checks, error codes, asynchrony) is as for attn_fwd; ATTN_ERR_NULL_PTR also covers a NULL
 * stride pointer, ATTN_ERR_MISALIGNED a stride that is not a multiple of 8.
 */
int attn_fwd_strided(const void *q, const void *k, const void *v, void *o, float *lse,
                     int B, int Hq, int Hkv, int Sq, int Sk, int D,
                     const long long *q_strides, const long long *k_strides,
                     const long long *v_strides, const long long *o_strides,
                     int causal, float scale, void *stream);

/*
 * attn_fwd with the workgroup shape of the tiled kernel forced, for tuning and for tests that run every shape
 * through both (the GEMM of the paper's Table 2 lists "tile-size specialization"; attention has the same knob):
 *   wg_rows = 256: 8 wavefronts x 32 query rows, one workgroup per compute unit, two wavefront groups half a
 *                  tile apart (the fastest steady state; what long sequences get);
 *   wg_rows = 128: 4 wavefronts x 32 query rows, two independent workgroups per compute unit (each hides the
 *                  other's start-up, drain and causal diagonal; what short sequences and small grids get);
 *   wg_rows = 0:   the library's own choice, i.e. exactly attn_fwd.
 * Any other value: ATTN_ERR_UNSUPPORTED.  Calls the 128-row kernel with 64-bit addressing serves (Sq <= 64, or a
 * head of K/V spanning 4 GiB or more) ignore wg_rows.  Everything else as for attn_fwd.
 */
int attn_fwd_tile(const void *q, const void *k, const void *v, void *o, float *lse,
                  int B, int Hq, int Hkv, int Sq, int Sk, int D,
                  int causal, float scale, int wg_rows, void *stream);

/* Static, never-freed description of a return code of this library. */
const char *attn_strerror(int code);

/* Library version, major*10000 + minor*100 + patch. */
int attn_version(void);

/*
 * Algorithmic FLOPs of one attn_fwd call: 4*D per visible (query, key) pair
 * (2*D for q.k and 2*D for p.v; softmax and masked pairs are not counted).
 * Host-only arithmetic, no GPU needed.  Returns -1 on bad dimensions.
 */
double attn_fwd_flops(int B, int Hq, int Hkv, int Sq, int Sk, int D, int causal);

/*
 * Measurement aid, no part of the method (the bench reports the published matrix peak AND what
 * this GPU sustains on nothing but matrix instructions): enqueue
 * `blocks` workgroups of 8 wavefronts that each issue 4*iters dense bf16 32x32x16 MFMAs and
 * nothing else.  Returns the FLOPs performed (time it with events on `stream`), or -1.0 on
 * bad arguments / refused launch.  `sink` is DEVICE memory of at least 4 bytes, never
 * written in practice.  Asynchronous, allocates nothing.
 */
double attn_mfma_calibration(float *sink, int blocks, int iters, void *stream);

/*
 * The same measurement with operands of a chosen kind.  The GPU runs against a power limit and the clock it
 * settles to under matrix load depends on how many operand bits toggle, so the rate the matrix pipe sustains is a
 * function of the data: data 0 = the smoothly varying positive operands of attn_mfma_calibration, 1 = all zeros
 * (what the pipe does when power is no limit), 2 = values with the spread of a standard normal, different per
 * lane, element and workgroup (the distribution of the benchmark inputs), 3 = the operands of 2 on the other
 * bf16 shape, v_mfma_f32_16x16x32_bf16 (every other kind and every kernel here use 32x32x16).  Kinds 1 and 2
 * issue 8*iters MFMAs per wavefront, kind 3 16*iters of the half-sized instruction: the same FLOPs, which the
 * return value counts.  Kinds 4 and 5 are kinds 3 and 2 with workgroups of 4 wavefronts, i.e. ONE wavefront per
 * SIMD instead of two: what a schedule sustains in which only one wavefront of a SIMD issues MFMAs at a time.
 * Same error behaviour; any other `data` returns -1.0.
 */
double attn_mfma_calibration_data(float *sink, int blocks, int iters, int data, void *stream);

/*
 * What the bench prices the kernels against, read from the HIP runtime rather than assumed (measurement aid, no
 * part of the method): the compute-unit count and the maximum shader clock (kHz) of HIP device `device`, and the
 * dense bf16 matrix peak that follows from them, cus * 4096 flop per clock * clock, in TFLOP/s (a CDNA4 compute
 * unit retires 4 x 1024 bf16 multiply-add flops per clock on its four matrix cores).  Any of the three output
 * pointers may be NULL.  Host memory, host call; touches no stream.  Returns ATTN_OK, ATTN_ERR_BAD_SHAPE for a
 * negative device index, or ATTN_ERR_LAUNCH if the runtime has no such device.
 */
int attn_device_info(int device, int *cus, int *clock_khz, double *bf16_peak_tflops);

#ifdef __cplusplus
}
#endif
#endif /* ATTN_MI355X_H */

/*
 * moe.h -- C ABI of the MI355X (gfx950) fused mixture-of-experts feed-forward in block-quantized FP8.
 *
 * Operation (the fused-MoE workload of the paper's Evaluation, "Kernel Performance": the block-quantized
 * FP8 configuration of DeepSeek-V3.2, model dimension H, intermediate dimension I, top-k routing, the experts
 * of one GPU under expert parallelism; same subsection, "Fused MoE" paragraph: tokens are routed through
 * sorted expert maps, blockwise quantization is preserved, the up-projection intermediates are
 * quantized to FP8 so that both projections run on the FP8 matrix cores).  For every token t and
 * routing slot k whose expert e = ids[t][k] is local (0 <= e < E):
 *
 *     xq, xs   = quant128(x[t])                       activation: per group of 128 features
 *     g_j, u_j = block-scaled dot products of xq with rows j and I+j of w13[e]        j < I
 *     a_j      = g_j / (1 + exp(-g_j)) * u_j          SiLU gate
 *     aq, as   = quant128(a)
 *     o_c      = block-scaled dot products of aq with row c of w2[e]                  c < H
 *     y[t][c]  = sum over local slots k (ascending) of wts[t][k] * o_c               bf16, rounded once
 *
 * quant128(v): per 128 consecutive values, scale = max|v| * (1/448) (1 if all zero), code =
 * e4m3(clamp(v * (1/scale), +-448)), every step in fp32, round to nearest even.  A block-scaled dot
 * product is  sum over 128-blocks b of (activation scale of b) * (weight scale of the row's 128-row
 * block and b) * (sum over the block of code values), accumulated in fp32.  FP8 is OCP e4m3.
 * Slots whose id is negative or >= E belong to other GPUs and contribute nothing; a token with no
 * local slot gets y = 0.
 *
 * DEVICE pointers, caller-owned, contiguous row-major:
 *     x   bf16 [T, H]            ids  int32 [T, KTOP]        wts  fp32 [T, KTOP]
 *     w13 e4m3 [E, 2I, H]        s13  fp32 [E, 2I/128, H/128]      (gate rows first, then up rows)
 *     w2  e4m3 [E, H, I]         s2   fp32 [E, H/128, I/128]
 *     y   bf16 [T, H]  (written)
 *     workspace: at least moe_ffn_fp8_workspace_bytes(...) bytes, 256-byte aligned; contents need
 *                not be initialised and are garbage afterwards.  The library allocates nothing.
 * x, w13, w2, y, workspace must be 16-byte aligned; ids, wts, s13, s2 4-byte aligned.
 *
 * Supported: H, I multiples of 128, at most 16384; 1 <= E <= 256;
 * 1 <= KTOP <= 16; 1 <= T, T*KTOP <= 2^20, T*H < 2^32 and T*KTOP*I < 2^32.  Inputs must be finite.
 *
 * `stream` is a hipStream_t passed as void* (NULL = the default stream): the call enqueues its
 * kernels there and returns.  Calls that share a workspace must not overlap.  Every argument
 * check precedes the first HIP call.  Return codes are those of attn.h: NULL_PTR, BAD_SHAPE
 * (a dimension out of range, workspace too small), MISALIGNED, LAUNCH.
 */
#ifndef MOE_MI355X_H
#define MOE_MI355X_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Bytes of workspace moe_ffn_fp8 needs for these sizes (0 if they are not supported). Host only. */
size_t moe_ffn_fp8_workspace_bytes(int T, int H, int I, int E, int KTOP);

int moe_ffn_fp8(const void *x, const int *ids, const float *wts,
                const void *w13, const float *s13, const void *w2, const float *s2,
                void *y, int T, int H, int I, int E, int KTOP,
                void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same path with two choices opened up, for profiling, tuning and tests:
 *   first_stage..last_stage  run only these stages (0 routing, 1 activation quantization, 2 gate/up product
 *       with SiLU and requantization, 3 down product, 4 combine); the stages before first_stage must have run
 *       on the same arguments, workspace and row_tile.  moe_ffn_fp8 is 0..4.
 *   row_tile  rows of one expert per workgroup of the two products: 64, 128, or 0 = what moe_ffn_fp8 does (128).
 *       An expert's rows are cut into tiles of row_tile rows and a remainder (an expert with row_tile + 1 ..
 *       row_tile + 32 rows gets a single tile); every tile runs the 64-, 128- or 160-row code that fits its rows.
 * A stage range outside 0..4 or another row_tile: ATTN_ERR_UNSUPPORTED.
 */
int moe_ffn_fp8_ex(const void *x, const int *ids, const float *wts,
                   const void *w13, const float *s13, const void *w2, const float *s2,
                   void *y, int T, int H, int I, int E, int KTOP,
                   void *workspace, size_t workspace_bytes,
                   int first_stage, int last_stage, int row_tile, void *stream);

/*
 * moe_ffn_fp8 for callers that cannot allocate device memory and so have no workspace to pass: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, arguments, checks and
 * results as moe_ffn_fp8 (bit for bit: the same kernels run), but the scratch memory is a device array that is
 * part of the library's code object: MOE_FFN_FP8_STATIC_MAX_BYTES bytes on every GPU the library runs on, held
 * until the process ends.  The call allocates and frees nothing (no hipMalloc, no hipFree, no allocating library
 * routine); the first call on a device looks the array's address up once (hipGetSymbolAddress) and keeps it.
 * Sizes whose moe_ffn_fp8_workspace_bytes(T, H, I, E, KTOP) exceeds MOE_FFN_FP8_STATIC_MAX_BYTES are rejected with
 * ATTN_ERR_TOO_LARGE and nothing is launched (the paper's configuration, H = 7168, I = 2048, top-4 of 32 local
 * experts, fits up to T = 1024 tokens).  Every call on one GPU uses that GPU's one array, which keeps whatever the
 * last call left there; nothing in it needs to start at zero (the first kernel rewrites every table it reads).
 * Calls that overlap on one GPU -- from two streams or two threads -- race on it: serialise them, or give all
 * but one a workspace of their own through moe_ffn_fp8.  ATTN_ERR_LAUNCH also covers a failed address lookup.
 */
#define MOE_FFN_FP8_STATIC_MAX_BYTES (128u << 20)
int moe_ffn_fp8_static(const void *x, const int *ids, const float *wts,
                       const void *w13, const float *s13, const void *w2, const float *s2,
                       void *y, int T, int H, int I, int E, int KTOP, void *stream);

/*
 * Where the parts of the workspace lie after a call (byte offset, or -1 for unsupported sizes or an
 * unknown part), for debugging and for tests that check the stages of the path one by one.  Rows are
 * in expert order; within an expert their order is not specified.  Parts:
 *   0 offsets    int32 [E+1]      first row of each expert (offsets[E] = number of local slots)
 *   6 sorted_tok int32 [T*KTOP]   token of each row            7 pos  int32 [T*KTOP]  row of slot (t,k) or -1
 *   8 xq         e4m3  [T, H]     quantized activations        9 xs   fp32 [T, H/128] their scales
 *                (both only for tokens that have a local slot)
 *  10 aq         e4m3  [rows, I]  quantized intermediate      11 as   fp32 [rows, I/128]
 *  12 o          fp32  [rows, H]  down-projection rows of tokens with two or more local slots (the row of a token
 *                with a single local slot goes straight to y as wts * row, which is all its sum has; its o is not written)
 * (1-5 are internal scheduling tables.)  Host only.
 */
long long moe_ffn_fp8_workspace_offset(int T, int H, int I, int E, int KTOP, int part);

/* Row tiles (workgroups per column tile) an expert with `rows` routed rows is cut into for row_tile = 0, 64 or
 * 128 as in moe_ffn_fp8_ex: tiles of row_tile rows and a remainder, except that an expert with row_tile + 1 ..
 * row_tile + 32 rows gets a single tile.  -1 for a negative count or another row_tile.  Host-only helper. */
int moe_ffn_fp8_row_tiles(int rows, int row_tile);

/* Algorithmic FLOPs per routed (token, local expert) pair: 2 * (2I*H + H*I).  Host-only helper. */
double moe_ffn_fp8_flops_per_pair(int H, int I);

#ifdef __cplusplus
}
#endif
#endif

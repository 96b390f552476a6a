// Fused mixture-of-experts feed-forward in block-quantized FP8 for gfx950 (MI355X): the
// paper's fused-MoE workload (Evaluation, "Kernel Performance", "Fused MoE" paragraph: tokens and experts are
// partitioned, tokens reach their experts through sorted maps, blockwise quantization is
// preserved, the up-projection intermediates are quantized to FP8 so that both projections run
// on the FP8 matrix cores).
//
// Five stages in four kernels on one stream, all state in the caller's workspace:
//   moe_prepare   workgroup 0: counting sort of the local (token, slot) pairs by expert (sorted
//                 rows, the inverse map, one record per row tile); the other workgroups: activation
//                 quantization, eight groups of 128 features per 32 lanes;
//   moe_gemm<UP>  per (row tile, 128 intermediate columns): gate and up products on
//                 v_mfma_scale_f32_32x32x64_f8f6f4, block scales applied per 128-deep stage,
//                 SiLU gate, requantization of the 128-column group, FP8 store;
//   moe_gemm<DN>  per (row tile, 256 output columns, or 128 if that is what it takes to give every CU a
//                 workgroup): down product; the row of a token with a single local slot
//                 goes straight to y (weight * row, rounded once), the others as fp32 rows to the workspace;
//   moe_combine   y[t] = sum over local slots of weight * row, rounded once to bf16, for the tokens with
//                 two or more local slots; zeros for those with none.
// With 16 to 256 rows per expert the products are bound by streaming the expert weights from
// HBM (each byte is used for 2 x rows FLOPs), so the grouped product keeps three 40-52 KB stages
// of direct-to-LDS copies per workgroup, two of them in flight, and does nothing clever with the MFMAs.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_layout.h"
#include <mutex>

#include "moe_launch.h"
#include "gfx950_prims.h"

namespace {

using namespace gfx950;

using namespace gemm_layout;   // kt_*: the 128-byte-row swizzled tile of the bf16 GEMM, here 128 e4m3 per row

// quant128 on four values of a 32-lane group: returns the four e4m3 codes packed little-endian.
// scale = amax * (1/448) (1 if amax = 0), code = e4m3(clamp(v * (1/scale))): fp32 throughout, a true
// division, v_cvt_pk_fp8_f32 rounds to nearest even (checked against the format on the device).
__device__ __forceinline__ float quant_scale(float amax) { return amax == 0.0f ? 1.0f : amax * (1.0f / 448.0f); }
__device__ __forceinline__ unsigned quant_pack4(float v0, float v1, float v2, float v3, float inv) {
    const float c0 = fminf(fmaxf(v0 * inv, -448.0f), 448.0f), c1 = fminf(fmaxf(v1 * inv, -448.0f), 448.0f);
    const float c2 = fminf(fmaxf(v2 * inv, -448.0f), 448.0f), c3 = fminf(fmaxf(v3 * inv, -448.0f), 448.0f);
    int p = __builtin_amdgcn_cvt_pk_fp8_f32(c0, c1, 0, false);
    p = __builtin_amdgcn_cvt_pk_fp8_f32(c2, c3, p, true);
    return (unsigned)p;
}

// ------------------------------------------------------------------------------------
// Routing: one workgroup of 16 wavefronts.  Thousands of slots land on a few dozen counters, so each
// wavefront counts into a histogram of its own (LDS atomics without a return value); the per-expert
// totals and the wavefronts' shares are turned into start rows by a block-wide scan; the scatter
// pass takes its row from the wavefront's own counter again, so only lanes of one wavefront ever
// contend.  Rows within an expert come out in no particular order: every row is computed on its
// own and found again through `pos`.
// ------------------------------------------------------------------------------------
__device__ __forceinline__ void route_block(const MoeParams& p) {
    __shared__ int wcnt[16 * 256];          // [wavefront][expert]: counts, then running row cursors
    __shared__ int rows_scan[256], tiles_scan[256], cnt[256];
    const int tid = threadIdx.x, wave = tid >> 6, E = p.E, n = p.T * p.KTOP;
    for (int i = tid; i < 16 * 256; i += 1024) wcnt[i] = 0;
    __syncthreads();
    // (both passes take kRU slots per thread and iteration with the loads issued together: this workgroup is
    // alone with the latency of its loads, and under the quantization blocks' traffic that latency is long)
    constexpr int kRU = 4;
    for (int i0 = tid; i0 < n; i0 += 1024 * kRU) {
        int e[kRU];
#pragma unroll
        for (int j = 0; j < kRU; ++j) { const int i = i0 + 1024 * j; e[j] = i < n ? p.ids[i] : -1; }
#pragma unroll
        for (int j = 0; j < kRU; ++j) if (e[j] >= 0 && e[j] < E) atomicAdd(&wcnt[wave * 256 + e[j]], 1);
    }
    __syncthreads();
    if (tid < 256) {                         // expert tid: total, and each wavefront's offset inside the expert
        int run = 0;
        if (tid < E)
            for (int w = 0; w < 16; ++w) { const int c = wcnt[w * 256 + tid]; wcnt[w * 256 + tid] = run; run += c; }
        cnt[tid] = run;
        rows_scan[tid] = run;
        tiles_scan[tid] = moe_row_tiles(run, p.bm);
    }
    __syncthreads();
    for (int d = 1; d < 256; d <<= 1) {      // inclusive scans over the experts
        int r = 0, t = 0;
        if (tid < 256 && tid >= d) { r = rows_scan[tid - d]; t = tiles_scan[tid - d]; }
        __syncthreads();
        if (tid < 256) { rows_scan[tid] += r; tiles_scan[tid] += t; }
        __syncthreads();
    }
    if (tid < E) {
        const int nt = moe_row_tiles(cnt[tid], p.bm);
        const int start = rows_scan[tid] - cnt[tid], tstart = tiles_scan[tid] - nt;
        p.offsets[tid] = start;
        for (int w = 0; w < 16; ++w) wcnt[w * 256 + tid] += start;
        for (int m = 0; m < nt; ++m) {
            p.tile_rec[tstart + m] = MoeTileRec{tid, start, cnt[tid], tstart};
        }
        if (tid == E - 1) { p.offsets[E] = rows_scan[tid]; p.ntiles[0] = tiles_scan[tid]; }
    }
    __syncthreads();
    for (int i0 = tid; i0 < n; i0 += 1024 * kRU) {
        int e[kRU];
#pragma unroll
        for (int j = 0; j < kRU; ++j) { const int i = i0 + 1024 * j; e[j] = i < n ? p.ids[i] : -1; }
#pragma unroll
        for (int j = 0; j < kRU; ++j) {
            const int i = i0 + 1024 * j;
            if (i >= n) break;
            int r = -1;
            if (e[j] >= 0 && e[j] < E) {
                r = atomicAdd(&wcnt[wave * 256 + e[j]], 1);
                p.sorted_tok[r] = i / p.KTOP;
            }
            p.pos[i] = r;
        }
    }
}

// ------------------------------------------------------------------------------------
// Activation quantization: 32 lanes per group of 128 features, 4 features per lane.
// ------------------------------------------------------------------------------------
constexpr int kMoeQuantGroups = 8;           // groups of 128 features one 32-lane unit quantizes, all loaded up front (4: 15 % slower)
__device__ __forceinline__ void quant_x_block(const MoeParams& p, unsigned block) {
    // 32 lanes take kQG consecutive groups of one token (all loads issued before the first use)
    constexpr int kQG = kMoeQuantGroups;
    const int gpt = p.H / 128;                                    // groups per token
    const int cpt = (gpt + kQG - 1) / kQG;                        // 32-lane work items per token
    const long long item = (long long)block * 32 + (threadIdx.x >> 5);
    if (item >= (long long)p.T * cpt) return;
    const int t = (int)(item / cpt), g0 = (int)(item - (long long)t * cpt) * kQG;
    {   // tokens without a local slot are never read by the products: skip them
        bool local = false;
        for (int k = 0; k < p.KTOP; ++k) { const int e = p.ids[t * p.KTOP + k]; local |= (e >= 0 && e < p.E); }
        if (!local) return;
    }
    const int l = threadIdx.x & 31;
    u32x2 raw[kQG];
#pragma unroll
    for (int q = 0; q < kQG; ++q) raw[q] = *(const u32x2*)(p.x + ((size_t)t * gpt + min(g0 + q, gpt - 1)) * 128 + l * 4);
#pragma unroll
    for (int q = 0; q < kQG; ++q) {
        if (g0 + q >= gpt) break;
        const size_t g = (size_t)t * gpt + g0 + q;
        const float v0 = __uint_as_float(raw[q][0] << 16), v1 = __uint_as_float(raw[q][0] & 0xffff0000u);
        const float v2 = __uint_as_float(raw[q][1] << 16), v3 = __uint_as_float(raw[q][1] & 0xffff0000u);
        float amax = fmaxf(fmaxf(fabsf(v0), fabsf(v1)), fmaxf(fabsf(v2), fabsf(v3)));
#pragma unroll
        for (int off = 16; off >= 1; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 32));
        const float scale = quant_scale(amax);
        const float inv = 1.0f / scale;
        *(unsigned*)(p.xq + g * 128 + l * 4) = quant_pack4(v0, v1, v2, v3, inv);
        if (l == 0) p.xs[g] = scale;
    }
}

// Stages 0 and 1 do not depend on each other: one launch, workgroup 0 routes while the others quantize.
// `stages` bit 0: routing, bit 1: quantization.
__global__ __launch_bounds__(1024) void moe_prepare(MoeParams p, int stages) {
    if (blockIdx.x == 0) {
        if (stages & 1) route_block(p);
    } else if (stages & 2) {
        quant_x_block(p, blockIdx.x - 1);
    }
}

// ------------------------------------------------------------------------------------
// Grouped block-scaled FP8 product.  Workgroup = 8 wavefronts = 4 (n) x 2 (m) for the MFMAs: 256 weight rows x
// BM routed rows.  An expert's rows are cut into tiles of p.bm (128 unless the caller asks for 64) and a
// remainder (moe_row_tiles: an expert with bm + 1 .. bm + 32 rows gets one tile); each workgroup picks
// the code for BM = 64, 128 or 160 from the rows its tile really has.
// Wavefront (wn, wm): weight rows 64 wn .. +63 as two 32-row MFMA operands, routed rows
// (BM/2) wm .. in the lanes, BM/64 blocks of 32 (transposed product, as in the bf16 GEMM).
//   UP:  the 256 weight rows of column tile nt are, per wavefront, 32 gate rows j and the 32 up
//        rows I + j of the same j: both accumulators of a lane meet the same (row, j).
//   DN:  256 consecutive rows of w2.
// One stage = 128 bytes of k for all rows (BM x 128 routed + 32 KB weights) plus the stage's row
// scales (dword copies); three stages in LDS; per stage two K = 64 MFMAs per operand pair into a fresh
// partial, then acc += partial * (row scale) * (weight block scale).  BM = 160: five 32-row blocks, three
// for the wavefronts wm = 0 and two for wm = 1.
// ------------------------------------------------------------------------------------
constexpr int kMoeBN = 256;
constexpr int kMoeLdsBytes = 3 * (160 * 128 + kMoeBN * 128);   // the largest stage set: three stages of BM = 160
constexpr int kMoeSaBytes = 8 * 128;                          // row scales per stage: 8 row groups x 32 dwords
constexpr int kMoeMaxKB = 128;                      // 128-blocks along k: H, I <= 16384

typedef __attribute__((address_space(3))) char* LdsChar;      // LDS pointers stay typed as such: a generic pointer would
typedef __attribute__((address_space(3))) float* LdsFloat;    // turn the scale reads into flat loads, which count as vector memory
template <bool UP, int BM, int BN>
__device__ __forceinline__ void moe_gemm_tile(const MoeParams& p, int e, int row0, int rows, int nt, LdsChar smem, LdsFloat sa_stage, LdsFloat sb_tab) {
    static_assert(BN == 256 || (BN == 128 && !UP), "the gate/up product pairs two 32-row weight blocks per wavefront");
    constexpr int NS = 3;                           // LDS stages
    constexpr int NIN = BN / 128;                   // 32-row weight blocks per wavefront (wavefront wn: weight rows 32 NIN wn ..)
    constexpr int NCB = BN / 32;                    // copy instructions of the weights per copying wavefront and stage
    constexpr int kStageA = BM * 128, kStageB = BN * 128, kStage = kStageA + kStageB;
    static_assert(NS * kStage <= kMoeLdsBytes, "stages exceed the workgroup's LDS");
    constexpr int NCA = BM / 32;                    // copy instructions of the routed rows per copying wavefront and stage
    constexpr int kW0 = BM == 160 ? 96 : BM / 2;    // routed rows of the wavefronts wm = 0; wm = 1 takes the rest
    constexpr int MB = BM == 160 ? 3 : BM / 64;     // 32-row blocks of routed rows per wavefront (BM = 160: the third only for wm = 0)
    constexpr int RPW = BM / 8;                     // routed rows per row group: a group's scales are one dword copy per stage
    static_assert(RPW <= 32, "a row group's scales fill at most the 32 dwords of its slot");
    constexpr int kCopies = NCA + NCB + 2;          // vmem operations per copying wavefront and stage
    // s_waitcnt immediate for vmcnt((NS - 2) kCopies), lgkmcnt(0): vmcnt's low four bits, then its two high bits at 14
    constexpr int kLater = (NS - 2) * kCopies;
    constexpr int kWaitNext = 0x0070 | (kLater & 15) | ((kLater >> 4) << 14);
    constexpr int kSaBytes = kMoeSaBytes;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave & 3, wm = wave >> 2;
    const int half = lane >> 5;

    const int KB = UP ? p.H : p.I;                  // bytes (= elements) per row of both operands
    const int nK = KB >> 7;
    const unsigned lds_base = (unsigned)(size_t)LDS_PTR(char, smem);

    // ---- copies: wavefronts 0-3 (one per SIMD) issue them: per stage instructions c + 4 n of the
    // routed rows (n < NCA) and of the weights (n < NCB), and the dword copies of the row scales for
    // the row groups c and c + 4.  Wavefronts 4-7 issue no memory traffic in the loop: four issuers
    // measured 5-10 % faster than eight.  (An L2 warm-up by the idle wavefronts, as in the bf16 GEMM,
    // was tried and is harmful here: an XCD's L2 holds 128 KB per CU, less than the LDS stages
    // already in flight, so lines touched early are evicted before the copies ask for them.) ----
    const bool copier = wave < 4;
    const int c4 = wave & 3;
    unsigned a_off[NCA], b_off[NCB], s_off[2];
    {
#pragma unroll
        for (int n = 0; n < NCA; ++n) {
            const int i = c4 + 4 * n;
            const int r = min(kt_dma_row(i, lane), rows - 1);         // rows past the tile re-read its last row
            const int src = UP ? p.sorted_tok[row0 + r] : row0 + r;
            a_off[n] = (unsigned)src * (unsigned)KB + 16u * (unsigned)kt_dma_chunk(i, lane);
        }
#pragma unroll
        for (int n = 0; n < NCB; ++n) {
            const int i = c4 + 4 * n, tr = kt_dma_row(i, lane);
            int wrow;
            if (UP) wrow = ((tr & 63) >> 5) * p.I + nt * 128 + ((tr >> 6) << 5) + (tr & 31);
            else wrow = min(nt * BN + tr, p.H - 1);                   // rows past H re-read the last one
            b_off[n] = (unsigned)wrow * (unsigned)KB + 16u * (unsigned)kt_dma_chunk(i, lane);
        }
#pragma unroll
        for (int n = 0; n < 2; ++n) {
            const int r = min(RPW * (c4 + 4 * n) + (lane % RPW), rows - 1);
            const int src = UP ? p.sorted_tok[row0 + r] : row0 + r;
            s_off[n] = 4u * (unsigned)src * (unsigned)nK;
        }
    }
    const char* const a_base = UP ? (const char*)p.xq : (const char*)p.aq;
    const char* const b_base = UP ? (const char*)(p.w13 + (size_t)e * 2 * (size_t)p.I * (size_t)p.H)
                                  : (const char*)(p.w2 + (size_t)e * (size_t)p.H * (size_t)p.I);
    const char* const s_base = UP ? (const char*)p.xs : (const char*)p.as;
    const unsigned lds_copy_base = lds_base + c4 * 1024;
    const unsigned sa_base = (unsigned)(size_t)LDS_PTR(float, sa_stage) + c4 * 128;
    auto dma_stage = [&](int U, auto sc) __attribute__((always_inline)) {
        constexpr int s = decltype(sc)::value;
        static_for<0, NCA>([&](auto n) __attribute__((always_inline)) {
            dma_to_lds_16B<s * kStage + n.value * 4096>(a_base + (size_t)U * 128, a_off[n.value], lds_copy_base);
        });
        static_for<0, NCB>([&](auto n) __attribute__((always_inline)) {
            dma_to_lds_16B<s * kStage + kStageA + n.value * 4096>(b_base + (size_t)U * 128, b_off[n.value], lds_copy_base);
        });
        if (lane < 32) {                            // a slot holds 32 dwords: the upper half of the wavefront stays out
            dma_to_lds_4B<s * kSaBytes>(s_base + (size_t)U * 4, s_off[0], sa_base);
            dma_to_lds_4B<s * kSaBytes + 512>(s_base + (size_t)U * 4, s_off[1], sa_base);
        }
    };

    // ---- weight block scales of all stages into LDS (read back as wavefront-uniform broadcasts; a
    // global load inside the loop would make the compiler wait for the copies in flight at every use) ----
    if (tid < 2 * nK) {
        const int which = tid / nK, b = tid - which * nK;
        const float* src;
        if (UP) src = p.s13 + ((size_t)e * 2 * (p.I >> 7) + (which ? (p.I >> 7) : 0) + nt) * nK;   // gate rows, up rows of block nt
        else src = p.s2 + ((size_t)e * (p.H >> 7) + min(nt * NIN + (NIN == 2 ? which : 0), (p.H >> 7) - 1)) * nK;
        sb_tab[which * kMoeMaxKB + b] = src[b];
    }
    const int sb_sel0 = UP ? 0 : (NIN == 2 ? wn >> 1 : 0), sb_sel1 = UP ? 1 : sb_sel0;

    // ---- per-lane LDS read addresses (stage 0): K = 64 operand = 32 bytes = chunks 4 ks + 2 half + {0,1} ----
    unsigned a_addr[2][2], b_addr[2][2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            a_addr[ks][q] = lds_base + kt_offset(kW0 * wm + (lane & 31), 4 * ks + 2 * half + q);
            b_addr[ks][q] = lds_base + kStageA + kt_offset(32 * NIN * wn + (lane & 31), 4 * ks + 2 * half + q);
        }
    // row scale of routed row m of the tile: dword m % RPW of row group m / RPW
    int sa_idx[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int m = min(kW0 * wm + 32 * mb + (lane & 31), BM - 1);     // (a block that does not exist reads a valid slot)
        sa_idx[mb] = (m / RPW) * 32 + (m % RPW);
    }
    auto frag = [&](unsigned addr0, unsigned addr1, int imm) __attribute__((always_inline)) -> i32x8 {
        const i32x4 lo = *LDS_PTR(i32x4, (size_t)(addr0 + imm));
        const i32x4 hi = *LDS_PTR(i32x4, (size_t)(addr1 + imm));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };

    f32x16 acc[NIN][MB];
#pragma unroll
    for (int in = 0; in < NIN; ++in)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[in][mb][r] = 0.0f;

    auto barrier = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- down product: where each row goes.  A row that is the only local slot of its token is that token's
    // whole sum and is written to y directly.  The lookup (row -> token -> its slots -> weight: three dependent
    // loads) is done here, before the loop, by the wavefronts that do not copy (a copying wavefront would have
    // to wait for it before it may issue its first copies): thread 256 + m takes row m and hands token and
    // weight over through LDS once the stage buffers are free, after the loop ----
    int look_tok = -1;
    float look_w = 0.0f;
    if constexpr (!UP) {
        const int m = tid - 256;
        if (m >= 0 && m < rows) {
            const int t = p.sorted_tok[row0 + m];
            int nlocal = 0, slot = 0;
            for (int k = 0; k < p.KTOP; ++k) {
                const int rk = p.pos[t * p.KTOP + k];
                nlocal += rk >= 0 ? 1 : 0;
                if (rk == row0 + m) slot = k;
            }
            if (nlocal == 1) { look_tok = t; look_w = p.wts[t * p.KTOP + slot]; }
        }
    }

    // ---- prologue: NS - 1 stages in flight ----
    if (copier) {
        dma_stage(0, IntC<0>{});
        if (NS > 2 && 1 < nK) dma_stage(1, IntC<1>{});
    }

    auto step = [&](int U, auto sc) __attribute__((always_inline)) {
        constexpr int s = decltype(sc)::value;
        // stage U has landed once at most the copies of the stages issued after it (NS - 2 of them) are outstanding
        if (!copier) __builtin_amdgcn_s_waitcnt(0xC07F);                 // lgkmcnt(0): nothing of its own in flight
        else if (NS > 2 && U + 1 < nK) __builtin_amdgcn_s_waitcnt(kWaitNext);   // vmcnt(kCopies), lgkmcnt(0)
        else __builtin_amdgcn_s_waitcnt(0x0070);                         // vmcnt(0), lgkmcnt(0)
        asm volatile("" ::: "memory");
        barrier();                                             // stage U visible; stage U-1's buffer is free
        if (copier && U + NS - 1 < nK) dma_stage(U + NS - 1, IntC<(s + NS - 1) % NS>{});
        const float sb0 = sb_tab[sb_sel0 * kMoeMaxKB + U], sb1 = sb_tab[sb_sel1 * kMoeMaxKB + U];
        const f32x16 zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
        i32x8 fb[NIN][2];
        static_for<0, NIN>([&](auto in) __attribute__((always_inline)) {
            fb[in.value][0] = frag(b_addr[0][0], b_addr[0][1], s * kStage + in.value * 4096);
            fb[in.value][1] = frag(b_addr[1][0], b_addr[1][1], s * kStage + in.value * 4096);
        });
        static_for<0, MB>([&](auto mb) __attribute__((always_inline)) {
            if (BM == 160 && mb.value == 2 && wm != 0) return;        // rows 160..191 do not exist
            const float sa = sa_stage[s * (kSaBytes / 4) + sa_idx[mb.value]];
            const i32x8 fa0 = frag(a_addr[0][0], a_addr[0][1], s * kStage + mb.value * 4096);
            const i32x8 fa1 = frag(a_addr[1][0], a_addr[1][1], s * kStage + mb.value * 4096);
            static_for<0, NIN>([&](auto in) __attribute__((always_inline)) {
                f32x16 part = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[in.value][0], fa0, zero, 0, 0, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
                part = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[in.value][1], fa1, part, 0, 0, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
                const float f = sa * (in.value == 0 ? sb0 : sb1);
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[in.value][mb.value][r] = fmaf(part[r], f, acc[in.value][mb.value][r]);
            });
        });
    };
    for (int U = 0;;) {
        step(U, IntC<0>{}); if (++U >= nK) break;
        step(U, IntC<1>{}); if (++U >= nK) break;
        if constexpr (NS > 2) { step(U, IntC<2>{}); if (++U >= nK) break; }
    }

    // result layout of a lane: register r of operand `in`, block mb is weight row 32 in + 8 (r/4) + 4 half + r%4
    // of the wavefront's 64, routed row (BM/2) wm + 32 mb + lane%32
    if constexpr (UP) {
        // SiLU gate, then quant128 over the tile's 128 columns of each routed row
        float h[MB][16], amax[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            amax[mb] = 0.0f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float g = acc[0][mb][r];
                h[mb][r] = g / (1.0f + __expf(-g)) * acc[1][mb][r];
                amax[mb] = fmaxf(amax[mb], fabsf(h[mb][r]));
            }
            // across the two halves of the wavefront (rows 4 half + ..)
            const u32x2 sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(amax[mb]), __float_as_uint(amax[mb]), false, false);
            const unsigned s0 = sw[0], s1 = sw[1];
            amax[mb] = fmaxf(__uint_as_float(s0), __uint_as_float(s1));
        }
        __builtin_amdgcn_s_waitcnt(0xC07F);
        barrier();                                             // every wavefront is done with the stage buffers
        const LdsFloat ex = (LdsFloat)smem;                        // [wm][mb][wn][32]
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            if (half == 0) ex[((wm * MB + mb) * 4 + wn) * 32 + (lane & 31)] = amax[mb];
        __builtin_amdgcn_s_waitcnt(0xC07F);
        barrier();
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            float am = amax[mb];
#pragma unroll
            for (int w = 0; w < 4; ++w) am = fmaxf(am, ex[((wm * MB + mb) * 4 + w) * 32 + (lane & 31)]);
            const float scale = quant_scale(am);
            const float inv = 1.0f / scale;
            const int m = kW0 * wm + 32 * mb + (lane & 31);
            if (m < rows) {
                uint8_t* const dst = p.aq + (size_t)(row0 + m) * p.I + nt * 128 + 32 * wn + 4 * half;
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4)
                    *(unsigned*)(dst + 8 * g4) = quant_pack4(h[mb][4 * g4], h[mb][4 * g4 + 1], h[mb][4 * g4 + 2], h[mb][4 * g4 + 3], inv);
                if (wn == 0 && half == 0) p.as[(size_t)(row0 + m) * (p.I >> 7) + nt] = scale;
            }
        }
    } else {
        // A row that is the only local slot of its token is that token's whole sum: weight * row, rounded once
        // to bf16, goes to y directly (bit for bit what the combine step computes from the fp32 row) and the
        // fp32 row is neither written nor read again.  Other rows go to the workspace for moe_combine.
        static_assert(BM <= 256, "one lookup thread per row");
        __builtin_amdgcn_s_waitcnt(0xC07F);
        barrier();                                             // every wavefront is done with the stage buffers
        const LdsFloat hand = (LdsFloat)smem;                  // [row][token bits, weight]
        if (tid >= 256 && tid - 256 < BM) { hand[2 * (tid - 256)] = __int_as_float(look_tok); hand[2 * (tid - 256) + 1] = look_w; }
        __builtin_amdgcn_s_waitcnt(0xC07F);
        barrier();
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int m = kW0 * wm + 32 * mb + (lane & 31);
            if (m < rows) {
                const int dst = __float_as_int(hand[2 * m]);
                const float w = hand[2 * m + 1];
#pragma unroll
                for (int in = 0; in < NIN; ++in)
#pragma unroll
                    for (int g4 = 0; g4 < 4; ++g4) {
                        const int c = nt * BN + 32 * NIN * wn + 32 * in + 8 * g4 + 4 * half;
                        if (c < p.H) {
                            const f32x4 v = {acc[in][mb][4 * g4], acc[in][mb][4 * g4 + 1], acc[in][mb][4 * g4 + 2], acc[in][mb][4 * g4 + 3]};
                            if (dst >= 0) {
                                const bf16x4 out = {(__bf16)fmaf(w, v[0], 0.0f), (__bf16)fmaf(w, v[1], 0.0f), (__bf16)fmaf(w, v[2], 0.0f), (__bf16)fmaf(w, v[3], 0.0f)};   // as moe_combine: 0 + w * v
                                *(bf16x4*)(p.y + (size_t)dst * p.H + c) = out;
                            } else {
                                *(f32x4*)(p.o + (size_t)(row0 + m) * p.H + c) = v;
                            }
                        }
                    }
            }
        }
    }
}

// Kernel: maps the workgroup to its (row tile, column tile) and runs the tile code that fits the tile's rows.
template <bool UP>
__global__ __launch_bounds__(512, 1) void moe_gemm(MoeParams p) {
    __shared__ __attribute__((aligned(16))) char smem[kMoeLdsBytes];
    __shared__ __attribute__((aligned(16))) float sa_stage[3 * kMoeSaBytes / 4];
    static_assert(kMoeLdsBytes + 3 * kMoeSaBytes + 2 * kMoeMaxKB * 4 <= 160 * 1024, "LDS budget");
    __shared__ float sb_tab[2 * kMoeMaxKB];          // weight block scale of the tile's two 128-row blocks and every stage

    // workgroup -> (row tile mt, column tile nt).  The grid has max_tiles * NT workgroups (a multiple of
    // 8), of which ntiles * NT are live; XCD x (= blockIdx % 8) takes the x-th eighth of the live logical
    // ids in order, so the ~32 workgroups resident on an XCD are neighbours.  Logical order: expert by
    // expert; inside an expert column tile by column tile, the expert's row tiles innermost: neighbours
    // share their weight tile (same nt) or their routed rows (same mt), which the XCD's L2 then
    // fetches once.
    // Down product: column tiles of 256 weight rows, or of 128 when the wide ones would not give every CU a
    // workgroup (few experts in use, or a small H: 8 experts of 4096 x 14336 make 128 wide tiles).  The host
    // sizes the grid for the narrow tiles when the problem is small enough for that to happen (p.dn_narrow_ok);
    // the choice itself needs the number of row tiles, known only here.  (With enough wide tiles the narrow ones
    // are 3-15 % slower: measured.)
    const int ntl = p.ntiles[0];
    const bool narrow = !UP && p.dn_narrow_ok && ntl * ((p.H + kMoeBN - 1) / kMoeBN) < 256;
    const int NT = UP ? (p.I >> 7) : narrow ? (p.H >> 7) : (p.H + kMoeBN - 1) / kMoeBN;
    const int live = ntl * NT, per_xcd = (live + 7) >> 3;
    const int bid = blockIdx.x;
    const int logical = (bid & 7) * per_xcd + (bid >> 3);
    if ((bid >> 3) >= per_xcd || logical >= live) return;   // uniform: before any barrier
    const MoeTileRec rec = p.tile_rec[logical / NT];             // the expert whose block of ids holds `logical`
    const int cnt = moe_row_tiles(rec.rows, p.bm);                // its row tiles; the last takes what is left: up to bm + 32 rows
    const int off = logical - rec.first * NT;                     // in [0, cnt * NT)
    const int nt = off / cnt, j = off - nt * cnt;                 // column tile, row tile within the expert
    const int e = rec.expert, row0 = rec.row0 + j * p.bm;
    const int rows = j == cnt - 1 ? rec.rows - j * p.bm : p.bm;   // uniform
    const LdsChar tiles = LDS_PTR(char, smem);
    const LdsFloat sa = LDS_PTR(float, sa_stage), sb = LDS_PTR(float, sb_tab);
    if constexpr (!UP) {
        if (narrow) {
            if (rows > 128) moe_gemm_tile<false, 160, 128>(p, e, row0, rows, nt, tiles, sa, sb);
            else if (rows > 64) moe_gemm_tile<false, 128, 128>(p, e, row0, rows, nt, tiles, sa, sb);
            else moe_gemm_tile<false, 64, 128>(p, e, row0, rows, nt, tiles, sa, sb);
            return;
        }
    }
    if (rows > 128) moe_gemm_tile<UP, 160, 256>(p, e, row0, rows, nt, tiles, sa, sb);
    else if (rows > 64) moe_gemm_tile<UP, 128, 256>(p, e, row0, rows, nt, tiles, sa, sb);
    else moe_gemm_tile<UP, 64, 256>(p, e, row0, rows, nt, tiles, sa, sb);
}

// ------------------------------------------------------------------------------------
// Combine: y[t][c] = sum over local slots k (ascending) of wts[t][k] * o[pos[t][k]][c], bf16.  Tokens with exactly
// one local slot were written by the down product.
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void moe_combine(MoeParams p) {
    const int cblocks = (p.H / 8 + 255) / 256;
    const int t = blockIdx.x / cblocks;
    const int c = ((blockIdx.x - t * cblocks) * 256 + threadIdx.x) * 8;
    if (c >= p.H) return;
    int nlocal = 0;
    for (int k = 0; k < p.KTOP; ++k) nlocal += p.pos[t * p.KTOP + k] >= 0 ? 1 : 0;
    if (nlocal == 1) return;
    float acc[8] = {};
    for (int k = 0; k < p.KTOP; ++k) {
        const int r = p.pos[t * p.KTOP + k];
        if (r < 0) continue;
        const float w = p.wts[t * p.KTOP + k];
        const f32x4 a = *(const f32x4*)(p.o + (size_t)r * p.H + c), b = *(const f32x4*)(p.o + (size_t)r * p.H + c + 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) { acc[i] = fmaf(w, a[i], acc[i]); acc[4 + i] = fmaf(w, b[i], acc[4 + i]); }
    }
    bf16x8 out;
#pragma unroll
    for (int i = 0; i < 8; ++i) out[i] = (__bf16)acc[i];
    *(bf16x8*)(p.y + (size_t)t * p.H + c) = out;
}

}  // namespace

// Scratch memory for callers that cannot allocate (graph capture, tight serving loops): one array per GPU, part
// of the code object, alive until the process ends.  In host code the array's NAME is only a handle for the
// symbol lookup below, never an address: every use of its memory goes through the pointer the lookup returned
// for the device at hand (each GPU holds its own copy at its own address).
static __device__ __align__(256) unsigned char moe_scratch_array[kMoeStaticScratchBytes];

void* moe_static_scratch(size_t* bytes) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* ptrs[kMaxDevices] = {};
    if (bytes) *bytes = kMoeStaticScratchBytes;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(moe_scratch_array)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return nullptr;
        }
        ptrs[dev] = ptr;
    }
    return ptrs[dev];
}

int moe_launch(const MoeParams& p, int first, int last, hipStream_t stream) {
    auto on = [&](int stage) { return first <= stage && stage <= last; };
    const long long items = (long long)p.T * ((p.H / 128 + kMoeQuantGroups - 1) / kMoeQuantGroups);   // quantization: kMoeQuantGroups groups of a token per 32 lanes
    if (on(0) || on(1))
        hipLaunchKernelGGL(moe_prepare, dim3(1 + (on(1) ? (unsigned)((items + 31) / 32) : 0u)), dim3(1024), 0, stream, p,
                           (on(0) ? 1 : 0) | (on(1) ? 2 : 0));
    auto grid8 = [](long long n) { return dim3((unsigned)((n + 7) / 8 * 8)); };   // the tile order wants a multiple of 8
    const dim3 g_up = grid8((long long)p.max_tiles * (p.I / 128)),
               g_dn = grid8((long long)p.max_tiles * (p.dn_narrow_ok ? p.H / 128 : (p.H + kMoeBN - 1) / kMoeBN));
    if (on(2)) hipLaunchKernelGGL((moe_gemm<true>), g_up, dim3(512), 0, stream, p);
    if (on(3)) hipLaunchKernelGGL((moe_gemm<false>), g_dn, dim3(512), 0, stream, p);
    if (on(4)) hipLaunchKernelGGL(moe_combine, dim3((unsigned)(((p.H / 8 + 255) / 256) * p.T)), dim3(256), 0, stream, p);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

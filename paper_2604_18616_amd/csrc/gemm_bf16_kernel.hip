// bf16 GEMM for gfx950 (MI355X): C = A B with fp32 accumulation on v_mfma_f32_16x16x32_bf16 or
// v_mfma_f32_32x32x16_bf16 (the GEMM workload of the paper's Evaluation, "Kernel Performance"; Table 2 names the ingredients: software
// pipelining, MFMA, asynchronous copies, bank-conflict-free LDS layouts, vectorised access,
// workgroup swizzling, guarded edge handling, explicit scheduling).
//
// Tiled kernel, described for its largest shape (the template parameter Tile gives the others: 192 x 256, 128 x 128
// and 64 x 64 tiles, two or four LDS stages, either MFMA instruction): one workgroup of 8 wavefronts owns a 256 x 256
// tile of C, wavefront (wm, wn) a 128 (m) x 64 (n) part of it as MFMA tiles of the TRANSPOSED product (rows = n,
// lanes = m), so that a lane ends up holding 4 consecutive n of one C row.  The 16x16x32 instruction does the same
// FLOPs in twice the instructions and takes less power per FLOP, which is what limits large products on this GPU;
// its sub-steps are the two m-halves of a 32-deep reduction step instead of 16-deep steps over the whole tile.  A and B stream through LDS
// in 64-deep k stages, copied HBM -> LDS by global_load_lds_dwordx4 (no staging registers) into
// XOR-swizzled tiles that the operand reads hit without bank conflicts.  B stored [K,N] is read
// through ds_read_b64_tr_b16, which delivers the k-major MFMA operand from the n-major tile.
//
// Pipeline per 64-deep stage U (two LDS stages, ONE workgroup barrier per stage):
//     operand reads of sub-step ks+1 are issued before the 8 MFMAs of sub-step ks;
//     the copies of stage U+1 are issued one or two at a time between them;
//     before the barrier a wavefront waits for its own reads of stage U (all four sub-steps)
//     and for its own copies of stage U+1; after it, it reads sub-step 0 of stage U+1 while
//     the MFMAs of sub-step 3 of stage U run.  The barrier therefore separates LDS read phases,
//     not MFMA phases, and the matrix pipe has work across it.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "gemm_layout.h"
#include "gemm_launch.h"
#include "gfx950_prims.h"

namespace {

using namespace gemm_layout;
using namespace gfx950;

// ------------------------------------------------------------------------------------
// Tiled kernel.  Requires: a, b, c 16-byte aligned; N, K, lda, ldb, ldc multiples of 8;
// lda, ldb < 2^22.  M, N need not be multiples of the tile (source rows are clamped, stores
// guarded); K need not be a multiple of 64 (KTAIL: pieces past K are fetched from a valid
// address and zeroed in LDS by the copying wavefront before they are published).
// ------------------------------------------------------------------------------------
template <class T, bool B_NK, bool KTAIL>
__global__ __launch_bounds__(T::kWaves * 64, T::kWaves >= 4 ? T::kPerCU : 1) void gemm_bf16_tiled(GemmParams p) {
    constexpr int kBM = T::BM, kBN = T::BN, kMB = T::kMB, kNB = T::kNB, kWaveM = T::kWaveM;
    constexpr int kStageA = T::kStageA, kStageB = T::kStageB, kBOffset = T::kBOffset;
    constexpr int kCopiers = T::kCopiers, kCopiesA = T::kCopiesA, kCopiesB = T::kCopiesB, RB = T::kNRowBytes;
    constexpr int kBK = T::BK, kKS = T::kKS, NS = T::NS, RBK = T::kRBK;
    constexpr bool MI16 = T::MI == 16;
    // blocks of the wavefront tile per MFMA shape: kRM x kRN result registers sets, kHalfM m-blocks per sub-step (MI16)
    constexpr int kRM = MI16 ? T::kWaveM / 16 : kMB, kRN = MI16 ? gemm_layout::kWaveN / 16 : kNB, kHalfM = kRM / 2;
    using Acc = std::conditional_t<MI16, f32x4, f32x16>;
    static_assert(kCopiesA <= kCopiesB, "the copy schedule pairs A with B instructions and ends with the B instructions left over");
    __shared__ __attribute__((aligned(16))) char smem[T::kLdsBytes + 256];   // stages, then the warm-up loads' sink

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % T::WM, wn = wave / T::WM;

    const TileCoord tc = tile_coord(blockIdx.x, gridDim.x, p.tiles_m, p.tiles_n);
    const int m0 = tc.tm * kBM, n0 = tc.tn * kBN;
    const int M = p.M, N = p.N, K = p.K;
    const int nK = (K + kBK - 1) / kBK;
    const unsigned lds_base = (unsigned)(size_t)LDS_PTR(char, smem);
    const unsigned a_rb = 2u * (unsigned)p.lda, b_rb = 2u * (unsigned)p.ldb;   // row pitches in bytes

    // ---- copies: wavefronts 0-3 (one per SIMD) issue them, instructions i = w + 4n (n = 0..7) of
    // each operand; wavefronts 4-7 do not copy (4 and 5 run the L2 warm-up below) ----
    const bool copier = wave < kCopiers;
    const int w4 = wave % kCopiers;
    unsigned a_off[kCopiesA], b_off[kCopiesB];   // per-lane source byte offsets relative to the stage's scalar base
#pragma unroll
    for (int n = 0; n < kCopiesA; ++n) {
        const int i = w4 + kCopiers * n;
        const int ra = min(m0 + kt_dma_row<RBK>(i, lane), M - 1) - m0;               // rows past M re-read row M-1
        a_off[n] = (unsigned)ra * a_rb + 16u * (unsigned)kt_dma_chunk<RBK>(i, lane);
    }
#pragma unroll
    for (int n = 0; n < kCopiesB; ++n) {
        const int i = w4 + kCopiers * n;
        if constexpr (B_NK) {
            const int rb = min(n0 + kt_dma_row<RBK>(i, lane), N - 1) - n0;
            b_off[n] = (unsigned)rb * b_rb + 16u * (unsigned)kt_dma_chunk<RBK>(i, lane);
        } else {
            const int col = min(n0 + 8 * nt_dma_chunk<RB, T::MI>(i, lane), N - 8) - n0;    // columns past N re-read the last piece
            b_off[n] = (unsigned)nt_dma_row<RB>(i, lane) * b_rb + 2u * (unsigned)col;
        }
    }
    const char* const a_base = (const char*)(p.a + (long long)m0 * p.lda);
    const char* const b_base = B_NK ? (const char*)(p.b + (long long)n0 * p.ldb) : (const char*)(p.b + n0);

    // one copy instruction: j < kCopiesA part j of A, else part j-kCopiesA of B, of stage U into LDS stage `buf`
    const unsigned lds_copy_base = lds_base + w4 * 1024;   // instruction i = w4 + kCopiers n lands at i * 1024
    auto dma = [&](int U, auto bufc, auto jc) __attribute__((always_inline)) {
        constexpr int buf = decltype(bufc)::value;
        constexpr int j = decltype(jc)::value;
        constexpr int n = j < kCopiesA ? j : j - kCopiesA;
        const int i = w4 + kCopiers * n;
        if constexpr (j < kCopiesA) {
            unsigned off = a_off[n];
            if constexpr (KTAIL)
                if (U == nK - 1 && U * kBK + 8 * kt_dma_chunk<RBK>(i, lane) >= K) off -= 16u * (unsigned)kt_dma_chunk<RBK>(i, lane);
            dma_to_lds_16B<buf * kStageA + n * kCopiers * 1024>(a_base + (size_t)U * (kBK * 2), off, lds_copy_base);
        } else if constexpr (B_NK) {
            unsigned off = b_off[n];
            if constexpr (KTAIL)
                if (U == nK - 1 && U * kBK + 8 * kt_dma_chunk<RBK>(i, lane) >= K) off -= 16u * (unsigned)kt_dma_chunk<RBK>(i, lane);
            dma_to_lds_16B<kBOffset + buf * kStageB + n * kCopiers * 1024>(b_base + (size_t)U * (kBK * 2), off, lds_copy_base);
        } else {
            unsigned off = b_off[n];
            if constexpr (KTAIL)
                if (U == nK - 1 && U * kBK + nt_dma_row<RB>(i, lane) >= K) off -= (unsigned)nt_dma_row<RB>(i, lane) * b_rb;
            dma_to_lds_16B<kBOffset + buf * kStageB + n * kCopiers * 1024>(b_base + (size_t)U * kBK * (size_t)b_rb, off, lds_copy_base);
        }
    };
    // K tail: zero what this wavefront copied from past K (both operands: 0 * garbage must be 0)
    auto zero_tail = [&](int U, int buf) __attribute__((always_inline)) {
        if constexpr (KTAIL) {
            if (U == nK - 1 && copier) {
#pragma unroll
                for (int n = 0; n < kCopiesA; ++n) {
                    const int i = w4 + kCopiers * n;
                    const unsigned dst = i * 1024 + lane * 16;
                    if (U * kBK + 8 * kt_dma_chunk<RBK>(i, lane) >= K) *(u32x4*)(smem + buf * kStageA + dst) = u32x4{0u, 0u, 0u, 0u};
                }
#pragma unroll
                for (int n = 0; n < kCopiesB; ++n) {
                    const int i = w4 + kCopiers * n;
                    const unsigned dst = i * 1024 + lane * 16;
                    const bool b_past = B_NK ? (U * kBK + 8 * kt_dma_chunk<RBK>(i, lane) >= K) : (U * kBK + nt_dma_row<RB>(i, lane) >= K);
                    if (b_past) *(u32x4*)(smem + kBOffset + buf * kStageB + dst) = u32x4{0u, 0u, 0u, 0u};
                }
            }
        }
    };

    // ---- per-lane LDS read addresses (stage 0; stage, block and sub-step offsets are immediates) ----
    // MI = 32: one address per 16-deep step; MI = 16: one per 32-deep step (entries 0 .. BK/32 - 1)
    unsigned a_addr[kKS];            // second MFMA operand (lanes = m), block jm adds jm * 32 (16) rows
    unsigned b_addr[B_NK ? kKS : 2 * kRN];
    if constexpr (MI16) {
#pragma unroll
        for (int ks = 0; ks < kBK / 32; ++ks) a_addr[ks] = lds_base + kt_offset<RBK>(kt16_row(wm * kRM, lane), kt16_chunk(ks, lane));
        if constexpr (B_NK) {
#pragma unroll
            for (int ks = 0; ks < kBK / 32; ++ks) b_addr[ks] = lds_base + kBOffset + kt_offset<RBK>(kt16_row(wn * kRN, lane), kt16_chunk(ks, lane));
        } else {
#pragma unroll
            for (int in = 0; in < kRN; ++in)
#pragma unroll
                for (int x = 0; x < 2; ++x) b_addr[2 * in + x] = lds_base + kBOffset + tr16_offset<RB>(wn * kRN + in, 0, x, lane);
        }
    } else {
#pragma unroll
        for (int ks = 0; ks < kKS; ++ks) a_addr[ks] = lds_base + kt_offset<RBK>(kt_row(wm * kMB, lane), kt_chunk(ks, lane));
        if constexpr (B_NK) {
#pragma unroll
            for (int ks = 0; ks < kKS; ++ks) b_addr[ks] = lds_base + kBOffset + kt_offset<RBK>(kt_row(wn * kNB, lane), kt_chunk(ks, lane));
        } else {
#pragma unroll
            for (int in = 0; in < kNB; ++in)
#pragma unroll
                for (int x = 0; x < 2; ++x) b_addr[2 * in + x] = lds_base + kBOffset + tr_offset<RB>(wn * kNB + in, 0, x, lane);
        }
    }

    // two operand sets.  MI = 32: sub-step ks (a 16-deep step) uses set ks & 1.  MI = 16: sub-step q covers the m-half
    // q & 1 of the 32-deep step q >> 1: its A blocks are in set q & 1, the B blocks of the step in the set given by the
    // parity of the step's number counted over the stage ring (consecutive steps alternate, also across stages).
    bf16x8 fa[2][MI16 ? kHalfM : kMB], fb[2][kRN];
    auto tr_pair = [&](unsigned addr_lo, unsigned addr_hi) __attribute__((always_inline)) {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, (size_t)addr_lo));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, (size_t)addr_hi));
        const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, v);
    };
    auto read_frags = [&](auto bufc, auto ksc) __attribute__((always_inline)) {
        constexpr int buf = decltype(bufc)::value, ks = decltype(ksc)::value, set = ks & 1;
        if constexpr (MI16) {
            constexpr int k32 = ks >> 1, mh = ks & 1, bset = (k32 + buf * (kBK / 32)) & 1;
            static_for<0, kHalfM>([&](auto j) __attribute__((always_inline)) {
                fa[set][j.value] = *LDS_PTR(bf16x8, (size_t)(a_addr[k32] + buf * kStageA + (mh * kHalfM + j.value) * 16 * RBK));
            });
            if constexpr (mh == 0)
                static_for<0, kRN>([&](auto in) __attribute__((always_inline)) {
                    if constexpr (B_NK) fb[bset][in.value] = *LDS_PTR(bf16x8, (size_t)(b_addr[k32] + buf * kStageB + in.value * 16 * RBK));
                    else fb[bset][in.value] = tr_pair(b_addr[2 * in.value] + buf * kStageB + k32 * 32 * RB,
                                                      b_addr[2 * in.value + 1] + buf * kStageB + k32 * 32 * RB);
                });
        } else {
            static_for<0, kMB>([&](auto jm) __attribute__((always_inline)) {
                fa[set][jm.value] = *LDS_PTR(bf16x8, (size_t)(a_addr[ks] + buf * kStageA + jm.value * 32 * RBK));
            });
            static_for<0, kNB>([&](auto in) __attribute__((always_inline)) {
                if constexpr (B_NK) fb[set][in.value] = *LDS_PTR(bf16x8, (size_t)(b_addr[ks] + buf * kStageB + in.value * 32 * RBK));
                else fb[set][in.value] = tr_pair(b_addr[2 * in.value] + buf * kStageB + ks * 16 * RB,
                                                 b_addr[2 * in.value + 1] + buf * kStageB + ks * 16 * RB);
            });
        }
    };

    Acc acc[kRN][kRM];
#pragma unroll
    for (int in = 0; in < kRN; ++in)
#pragma unroll
        for (int jm = 0; jm < kRM; ++jm)
#pragma unroll
            for (int r = 0; r < (MI16 ? 4 : 16); ++r) acc[in][jm][r] = 0.0f;

    // the MFMAs of sub-step q
    auto mfma_set = [&](auto bufc, auto qc) __attribute__((always_inline)) {
        constexpr int q = decltype(qc)::value, set = q & 1;
        if constexpr (MI16) {
            constexpr int mh = q & 1, bset = ((q >> 1) + decltype(bufc)::value * (kBK / 32)) & 1;
            static_for<0, kHalfM>([&](auto j) __attribute__((always_inline)) {
                static_for<0, kRN>([&](auto in) __attribute__((always_inline)) {
                    constexpr int jm = mh * kHalfM + j.value;
                    acc[in.value][jm] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[bset][in.value], fa[set][j.value], acc[in.value][jm], 0, 0, 0);
                });
            });
        } else {
            static_for<0, kMB>([&](auto jm) __attribute__((always_inline)) {
                static_for<0, kNB>([&](auto in) __attribute__((always_inline)) {
                    acc[in.value][jm.value] =
                        __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][in.value], fa[set][jm.value], acc[in.value][jm.value], 0, 0, 0);
                });
            });
        }
    };
    auto wait_all = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) and lgkmcnt(0): own copies landed, own LDS reads returned
        asm volatile("" ::: "memory");
    };
    auto barrier = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- L2 warm-up --------------------------------------------------------------------------
    // The workgroups that share an operand panel run in near lockstep, so a panel slice that is
    // not in L2 yet is missed by all of them at once and every one waits out the HBM latency, which
    // two LDS stages cannot cover.  kAhead stages early, one dword of each cache line of a stage
    // is touched so that the copy issued later finds its lines in L2.  The workgroups resident on
    // an XCD form GEMM_GM x 32/GEMM_GM patches of tiles (tile_coord): those that share an A panel each
    // touch their share of its 256 lines (wavefront 4), those that share a B panel likewise (wavefront 5),
    // which keeps the extra L2 -> L1 traffic at a fifth of the copies'.  Loads return in order, so
    // a wavefront that also copies would meet its warm-up loads again at its next wait for the
    // copies: wavefronts 4 and 5 issue no copies and wait for memory only once, at the end.  The
    // loaded dwords are never used: they go to a 256-byte LDS sink, so no register waits for them.
#ifndef GEMM_AHEAD
#define GEMM_AHEAD 3
#endif
#ifndef GEMM_EARLY
#define GEMM_EARLY 2
#endif
    constexpr int kEarly = GEMM_EARLY < kCopiesA ? GEMM_EARLY : kCopiesA;                 // copy pairs (A, B) issued in the first sub-step, the rest in the second
    constexpr int kAhead = GEMM_AHEAD;                 // 0 switches the warm-up off
    const int nK_whole = KTAIL ? nK - 1 : nK;          // stages that lie wholly inside K
    const bool warmer = kAhead > 0 && T::kWaves == 8 && NS == 2 && (wave == 4 || wave == 5);
    unsigned warm_off;
    constexpr int kShareA = 32 / GEMM_GM, kShareB = GEMM_GM;      // workgroups of an XCD's patch that read the same A / B panel
    static_assert(kBM / kShareA <= 64 && kBN / kShareB <= 64, "one warm-up instruction per wavefront");
    if (wave == 4) {
        const int r = (tc.tn % kShareA) * (kBM / kShareA) + lane % (kBM / kShareA);
        warm_off = (unsigned)(min(m0 + r, M - 1) - m0) * a_rb;
    } else {
        const int r = (tc.tm % kShareB) * (kBN / kShareB) + lane % (kBN / kShareB);
        if (B_NK) warm_off = (unsigned)(min(n0 + r, N - 1) - n0) * b_rb;
        else warm_off = (unsigned)(r >> 2) * b_rb + 2u * (unsigned)(min(n0 + 64 * (r & 3), N - 2) - n0);
    }
    const char* const warm_base = wave == 4 ? a_base : b_base;
    const size_t warm_step = (wave == 4 || B_NK) ? (size_t)(kBK * 2) : (size_t)kBK * (size_t)b_rb;
    auto warm = [&](int U) __attribute__((always_inline)) {
        const char* const src = warm_base + (size_t)U * warm_step;
        dma_to_lds_4B<0>(src, warm_off, lds_base + T::kLdsBytes);
    };

    // vmcnt(n) with lgkmcnt(0): n = copies of the stages that may still be in flight
    constexpr auto vm = [](int n) constexpr { return 0x0070 | (n & 15) | ((n >> 4) << 14); };
    constexpr int kPerStage = kCopiesA + kCopiesB;
    // wait until this wavefront's copies of stage X have landed, given that stages up to `issued` have been issued
    auto wait_stage = [&](int X, int issued) __attribute__((always_inline)) {
        if (copier) {
            const int later = min(issued, nK - 1) - X;              // stages issued after X
            if (NS > 3 && later >= 2) __builtin_amdgcn_s_waitcnt(vm(2 * kPerStage));
            else if (NS > 2 && later == 1) __builtin_amdgcn_s_waitcnt(vm(kPerStage));
            else __builtin_amdgcn_s_waitcnt(vm(0));
        } else {
            __builtin_amdgcn_s_waitcnt(0xC07F);                     // lgkmcnt(0) only: warm-up loads stay in flight
        }
        asm volatile("" ::: "memory");
    };
    static_assert(NS <= 4, "wait_stage counts at most two later stages");

    // ---- prologue: stages 0 .. NS-2 in flight, stage 0 landed ----
    if (copier) {
        static_for<0, NS - 1>([&](auto st) __attribute__((always_inline)) {
            if (st.value < nK) static_for<0, kPerStage>([&](auto j) __attribute__((always_inline)) { dma(st.value, st, j); });
        });
    } else if (warmer) {
        static_for<1, kAhead>([&](auto u) __attribute__((always_inline)) { if (u.value < nK_whole) warm(u.value); });
    }
    wait_stage(0, NS - 2);
    zero_tail(0, 0);
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): the zeros are written
    barrier();
    read_frags(IntC<0>{}, IntC<0>{});

    // one BK-deep stage U held in LDS stage BUF; the copies of stage U + NS - 1 go to the buffer stage U - 1 left
    auto step = [&](auto bufc, int U) __attribute__((always_inline)) {
        constexpr int BUF = decltype(bufc)::value;
        constexpr int NEXT = (BUF + 1) % NS, DST = (BUF + NS - 1) % NS;
        const bool more = U + 1 < nK, copy = U + NS - 1 < nK;
        static_for<0, kKS - 1>([&](auto ks) __attribute__((always_inline)) {
            read_frags(bufc, IntC<ks.value + 1>{});
            if constexpr (ks.value == 0) {
                constexpr int first = kKS > 2 ? 2 * kEarly : kPerStage;   // with two sub-steps everything goes here
                if (copier) {
                    if (copy) static_for<0, first>([&](auto n) __attribute__((always_inline)) {
                        dma(U + NS - 1, IntC<DST>{}, IntC<copy_order(n.value, kCopiesA)>{}); });
                } else if (warmer && U + kAhead < nK_whole) {
                    warm(U + kAhead);
                }
            }
            if constexpr (ks.value == 1) {
                if (copier && copy) static_for<2 * kEarly, kPerStage>([&](auto n) __attribute__((always_inline)) {
                    dma(U + NS - 1, IntC<DST>{}, IntC<copy_order(n.value, kCopiesA)>{}); });
            }
            mfma_set(bufc, ks);
        });
        if (more) {
            wait_stage(U + 1, U + NS - 1);          // stage U+1 landed, own LDS reads returned
            if constexpr (KTAIL) {
                if (U + 2 == nK) {                  // the stage about to be published is the partial one
                    zero_tail(U + 1, NEXT);
                    __builtin_amdgcn_s_waitcnt(0xC07F); // lgkmcnt(0): the zeros are written
                }
            }
            barrier();
            read_frags(IntC<NEXT>{}, IntC<0>{});
        }
        mfma_set(bufc, IntC<kKS - 1>{});
    };
    for (int U = 0;;) {
        bool done = false;
        static_for<0, NS>([&](auto st) __attribute__((always_inline)) {
            if (!done) { step(st, U); if (++U >= nK) done = true; }
        });
        if (done) break;
    }
    __builtin_amdgcn_s_waitcnt(0xC07F);
    barrier();                                      // every wavefront has read its last operands: the stages become the C staging area

    wait_all();                                     // the last warm-up loads have landed

    // ---- epilogue: C^T fragments -> bf16 -> this wavefront's 128 x 64 staging tile -> 16-byte stores ----
    // (no copy is in flight: the last stage was awaited before it was read)
    char* const stage = smem + wave * (kWaveM * 128);
    if constexpr (MI16) {
#pragma unroll
        for (int in = 0; in < kRN; ++in)
#pragma unroll
            for (int jm = 0; jm < kRM; ++jm) {
                const int m = jm * 16 + mfma16_rc(lane);
                const int n = in * 16 + mfma16_out_row(lane, 0);
                u32x2 v;
                v[0] = pack_bf16x2(acc[in][jm][0], acc[in][jm][1]);
                v[1] = pack_bf16x2(acc[in][jm][2], acc[in][jm][3]);
                *(u32x2*)(stage + c_stage_offset(m, n)) = v;
            }
    } else {
        const int half = lane >> 5;
#pragma unroll
        for (int in = 0; in < kNB; ++in)
#pragma unroll
            for (int jm = 0; jm < kMB; ++jm)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int m = jm * 32 + (lane & 31);
                    const int n = in * 32 + 8 * g + 4 * half;
                    u32x2 v;
                    v[0] = pack_bf16x2(acc[in][jm][4 * g + 0], acc[in][jm][4 * g + 1]);
                    v[1] = pack_bf16x2(acc[in][jm][4 * g + 2], acc[in][jm][4 * g + 3]);
                    *(u32x2*)(stage + c_stage_offset(m, n)) = v;
                }
    }
    __bf16* const ctile = p.c + (long long)(m0 + wm * kWaveM) * p.ldc + (n0 + wn * kWaveN);
#pragma unroll
    for (int it = 0; it < kWaveM / 8; ++it) {
        const int row = it * 8 + (lane >> 3);
        const int pos = lane & 7;
        const u32x4 val = *(const u32x4*)(stage + row * 128 + pos * 16);
        const int col = 8 * (pos ^ cswz(row));
        if (m0 + wm * kWaveM + row < M && n0 + wn * kWaveN + col < N)
            *(u32x4*)(ctile + (long long)row * p.ldc + col) = val;
    }
}

// ------------------------------------------------------------------------------------
// General kernel: any M, N, K, pitches and 2-byte-aligned pointers.  64 x 64 tile, 16-deep
// k steps through fp32 LDS tiles with zero fill past the edges, 4 x 4 outputs per thread,
// plain fp32 FMAs in k order.  Serves the shapes the tiled kernel's 16-byte pieces cannot.
// ------------------------------------------------------------------------------------
template <bool B_NK>
__global__ __launch_bounds__(256) void gemm_bf16_general(GemmParams p) {
    __shared__ float As[16][68];
    __shared__ float Bs[16][68];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int tm = blockIdx.x % p.tiles_m, tn = blockIdx.x / p.tiles_m;
    const int m0 = tm * 64, n0 = tn * 64;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < p.K; k0 += 16) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int idx = tid + 256 * t;
            {
                const int r = idx >> 4, kk = idx & 15;
                const bool ok = m0 + r < p.M && k0 + kk < p.K;
                As[kk][r] = ok ? (float)p.a[(long long)(m0 + r) * p.lda + (k0 + kk)] : 0.0f;
            }
            if constexpr (B_NK) {
                const int c = idx >> 4, kk = idx & 15;
                const bool ok = n0 + c < p.N && k0 + kk < p.K;
                Bs[kk][c] = ok ? (float)p.b[(long long)(n0 + c) * p.ldb + (k0 + kk)] : 0.0f;
            } else {
                const int kk = idx >> 6, c = idx & 63;
                const bool ok = n0 + c < p.N && k0 + kk < p.K;
                Bs[kk][c] = ok ? (float)p.b[(long long)(k0 + kk) * p.ldb + (n0 + c)] : 0.0f;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float av[4], bv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { av[i] = As[kk][ty * 4 + i]; bv[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (m < p.M && n < p.N) p.c[(long long)m * p.ldc + n] = (__bf16)acc[i][j];
        }
}

}  // namespace

template <class T>
static void launch_tiled(GemmParams p, int b_is_nk, hipStream_t stream) {
    p.tiles_m = (p.M + T::BM - 1) / T::BM;
    p.tiles_n = (p.N + T::BN - 1) / T::BN;
    const dim3 grid((unsigned)(p.tiles_m * p.tiles_n)), block(T::kWaves * 64);
    const bool ktail = (p.K % T::BK) != 0;
#define GEMM_LAUNCH_TILED(NK, KT) hipLaunchKernelGGL((gemm_bf16_tiled<T, NK, KT>), grid, block, 0, stream, p)
    if (b_is_nk) { if (ktail) GEMM_LAUNCH_TILED(true, true); else GEMM_LAUNCH_TILED(true, false); }
    else         { if (ktail) GEMM_LAUNCH_TILED(false, true); else GEMM_LAUNCH_TILED(false, false); }
#undef GEMM_LAUNCH_TILED
}

// Tile-size choice: the shape that promises the most throughput, estimated as (what the shape delivers when
// every CU has its fill of workgroups) x (how full the last round of workgroups leaves the chip) x (the share of
// the tiles' area that lies inside the result).  The first factor is measured on large squares (TFLOP/s: 256 x 256
// tiles on the 16x16x32 instruction 1420, 192 x 256 tiles on it 1300, 128 x 128 in two stages with two
// workgroups per CU 1150, in four stages with one per CU 880, 64 x 64 with two per CU 700); the second is
// tiles / (slots x rounds) with 256 CUs x workgroups per CU slots.  Checked against measurements on squares from
// 1024 to 6144 and on rectangles from 1024 x 4096 to 1024 x 16384 and 3000 x 5000: it picks the fastest of the
// five everywhere (a half-filled chip runs somewhat faster than the estimate, which never changed the order).
int gemm_auto_tile(int M, int N) {
    struct Shape { int tile, edge_m, edge_n, slots; double peak; };
    static const Shape shapes[5] = {{25616, 256, 256, 256, 1420.0}, {19216, 192, 256, 256, 1300.0}, {128, 128, 128, 512, 1150.0},
                                    {1284, 128, 128, 256, 880.0}, {64, 64, 64, 512, 700.0}};
    int best = 25616;
    double best_rate = -1.0;
    for (const Shape& sh : shapes) {
        const long long tiles = (long long)((M + sh.edge_m - 1) / sh.edge_m) * ((N + sh.edge_n - 1) / sh.edge_n);
        const long long rounds = (tiles + sh.slots - 1) / sh.slots;
        const double useful = (double)M * (double)N / ((double)tiles * sh.edge_m * sh.edge_n);   // edge tiles compute padding
        const double rate = sh.peak * useful * (double)tiles / (double)(rounds * sh.slots);
        if (rate > best_rate) { best_rate = rate; best = sh.tile; }
    }
    return best;
}

int gemm_launch(GemmParams p, int b_is_nk, bool tiled, int tile, hipStream_t stream) {
    if (tiled) {
        if (tile == 0) tile = gemm_auto_tile(p.M, p.N);
        if (tile == 2564) launch_tiled<TileLarge4>(p, b_is_nk, stream);
        else if (tile == 256) launch_tiled<TileLarge>(p, b_is_nk, stream);
        else if (tile == 64) launch_tiled<TileTiny>(p, b_is_nk, stream);
        else if (tile == 1284) launch_tiled<TileSmall4>(p, b_is_nk, stream);
        else if (tile == 25616) launch_tiled<TileLarge16>(p, b_is_nk, stream);
        else if (tile == 19216) launch_tiled<TileTall16>(p, b_is_nk, stream);
        else if (tile == 256416) launch_tiled<TileLarge4_16>(p, b_is_nk, stream);
        else if (tile == 12816) launch_tiled<TileSmall16>(p, b_is_nk, stream);
        else if (tile == 128416) launch_tiled<TileSmall4_16>(p, b_is_nk, stream);
        else if (tile == 6416) launch_tiled<TileTiny16>(p, b_is_nk, stream);
        else launch_tiled<TileSmall>(p, b_is_nk, stream);
    } else {
        p.tiles_m = (p.M + 63) / 64;
        p.tiles_n = (p.N + 63) / 64;
        const dim3 grid((unsigned)(p.tiles_m * p.tiles_n)), block(256);
        if (b_is_nk) hipLaunchKernelGGL((gemm_bf16_general<true>), grid, block, 0, stream, p);
        else         hipLaunchKernelGGL((gemm_bf16_general<false>), grid, block, 0, stream, p);
    }
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

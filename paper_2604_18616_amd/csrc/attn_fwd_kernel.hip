// Flash-attention forward for gfx950 (MI355X): tiled S^T = K Q^T and O^T += V^T P^T on
// bf16 MFMA with an fp32 online softmax (paper Section 2 for the method, Figure 1 for the
// tiling this re-designs: one wavefront owns 32 query rows, K/V stream through LDS in
// 64-key tiles, operands swapped so that a softmax row lives in one lane column).
//
// Differences from the paper's MI300X kernel that matter here:
//   * scores stay fp32 until after the softmax (the paper packs S to bf16 first);
//   * V^T comes from ds_read_b64_tr_b16 on a row-major V tile instead of a transpose
//     during staging;
//   * one 32x32x16 MFMA replaces the paper's pair of 32x32x8;
//   * an LSE output, a causal mask with tile skipping, and ragged-size handling.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_layout.h"
#include "attn_launch.h"

namespace {

using namespace attn_layout;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

#define LDS_PTR(T, p) ((T __attribute__((address_space(3)))*)(p))

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// two fp32 -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    f32x2 f = {lo, hi};
    bf16x2 b = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(unsigned, b);
}

// Exchange between lane l and lane l ^ 32.  v_permlane32_swap(a, b) returns
//   r0 = { a[0..31], b[0..31] },  r1 = { a[32..63], b[32..63] }     (verified on gfx950),
// so with b = a, (r0, r1) is (value held by the low-half lane, value held by the
// high-half lane) in every lane.  The two results are copied to scalars before any
// reinterpretation: a bit cast applied directly to a vector element reads element 0.
__device__ __forceinline__ void swap_halves(float x, float& lo, float& hi) {
    const unsigned a = __float_as_uint(x);
    const u32x2 r = __builtin_amdgcn_permlane32_swap(a, a, false, false);
    const unsigned r0 = r[0], r1 = r[1];
    lo = __uint_as_float(r0);
    hi = __uint_as_float(r1);
}
__device__ __forceinline__ float max_across_halves(float x) {
    float lo, hi;
    swap_halves(x, lo, hi);
    return fmaxf(lo, hi);
}
__device__ __forceinline__ float sum_across_halves(float x) {
    float lo, hi;
    swap_halves(x, lo, hi);
    return lo + hi;
}

// Workgroup id -> (batch, query head, query tile).  Workgroups are handed to the 8 XCDs
// round-robin, and each XCD has its own L2: give every XCD a contiguous range of the
// logical order, in which all query tiles of the gqa heads that share one kv head are
// neighbours, so that one XCD's resident workgroups stream the same K/V through its L2.
// Causal: heavy (late) query tiles first.
struct BlockCoord { int b, hq, hk, qt; };
template <bool CAUSAL>
__device__ __forceinline__ BlockCoord block_coord(int bid, int nblocks, int Hq, int Hkv, int nQt) {
    const int g = Hq / Hkv;
    const int per_xcd = nblocks >> 3;
    const int logical = (bid < per_xcd * 8) ? (bid & 7) * per_xcd + (bid >> 3) : bid;
    const int W = g * nQt;
    const int pair = logical / W, rem = logical - pair * W;
    const int ord = rem / g, hin = rem - ord * g;
    BlockCoord c;
    c.b = pair / Hkv;
    c.hk = pair - c.b * Hkv;
    c.hq = c.hk * g + hin;
    c.qt = CAUSAL ? nQt - 1 - ord : ord;
    return c;
}

// ------------------------------------------------------------------------------------
// Generic kernel: any Sq, Sk >= 1.  256 threads = 4 wavefronts x 32 query rows (Br = 128),
// Bc = 64.  K/V tiles are prefetched global -> registers (128-bit loads, zero fill past
// Sk) while the previous tile is being consumed, then written to a swizzled LDS tile.
// ------------------------------------------------------------------------------------
template <int D, bool CAUSAL>
__global__ __launch_bounds__(256, 2) void attn_fwd_generic(AttnParams p) {
    constexpr int CPR = D / 8;                 // 16-byte chunks per row
    constexpr int NST = kBc * CPR / 256;       // chunks per thread per tile and matrix
    constexpr int KS = D / 16;                 // reduction steps of S^T = K Q^T
    constexpr int DB = D / 32;                 // 32-row blocks of O^T
    constexpr int kBr = 128;

    __shared__ __attribute__((aligned(16))) char smem[2 * tile_bytes<D>()];
    char* const sK = smem;
    char* const sV = smem + tile_bytes<D>();

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int half = lane >> 5;

    const BlockCoord bc = block_coord<CAUSAL>(blockIdx.x, gridDim.x, p.Hq, p.Hkv, p.nQt);
    const int q0 = bc.qt * kBr;
    const int Sq = p.Sq, Sk = p.Sk;
    const int shift = Sk - Sq;                 // causal: key j visible to query i iff j <= i + shift

    const __bf16* qh = p.q + ((size_t)bc.b * p.Hq + bc.hq) * (size_t)Sq * D;
    const __bf16* kh = p.k + ((size_t)bc.b * p.Hkv + bc.hk) * (size_t)Sk * D;
    const __bf16* vh = p.v + ((size_t)bc.b * p.Hkv + bc.hk) * (size_t)Sk * D;

    // number of key tiles this workgroup visits
    int nT;
    {
        const int q_last = min(q0 + kBr - 1, Sq - 1);
        const int lim_max = CAUSAL ? min(Sk - 1, q_last + shift) : Sk - 1;
        nT = lim_max < 0 ? 0 : lim_max / kBc + 1;
    }

    // this lane's query row and the last key it may see
    const int wrow0 = q0 + wave * kWaveRows;
    const int qi = wrow0 + (lane & 31);
    const int lim = CAUSAL ? min(Sk - 1, qi + shift) : Sk - 1;
    const int wave_lim_min = CAUSAL ? min(Sk - 1, wrow0 + shift) : Sk - 1;
    const int wave_lim_max = CAUSAL ? min(Sk - 1, wrow0 + kWaveRows - 1 + shift) : Sk - 1;

    // Q^T B-operand fragments: Q[qi][16*ks + 8*half .. +7], rows past Sq clamped (never stored)
    bf16x8 qf[KS];
    {
        const __bf16* qrow = qh + (size_t)min(qi, Sq - 1) * D + 8 * half;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = *(const bf16x8*)(qrow + 16 * ks);
    }

    f32x16 oacc[DB];
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;
    float m_run = -INFINITY;   // running max of the raw (unscaled) scores of this query row
    float l_run = 0.f;         // running sum over THIS lane's keys only (halves merged at the end)
    const float c = p.scale_log2;

    // staging registers
    u32x4 kreg[NST], vreg[NST];
    auto load_tile = [&](int t) {
#pragma unroll
        for (int n = 0; n < NST; ++n) {
            const int idx = n * 256 + tid;
            const int row = idx / CPR, ch = idx % CPR;
            const int key = t * kBc + row;
            if (key < Sk) {
                kreg[n] = *(const u32x4*)(kh + (size_t)key * D + ch * 8);
                vreg[n] = *(const u32x4*)(vh + (size_t)key * D + ch * 8);
            } else {
                kreg[n] = u32x4{0, 0, 0, 0};
                vreg[n] = u32x4{0, 0, 0, 0};
            }
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int n = 0; n < NST; ++n) {
            const int idx = n * 256 + tid;
            const int row = idx / CPR, ch = idx % CPR;
            *(u32x4*)(sK + k_chunk_offset<D>(row, ch)) = kreg[n];
            *(u32x4*)(sV + v_chunk_offset<D>(row, ch)) = vreg[n];
        }
    };

    if (nT > 0) load_tile(0);

    for (int t = 0; t < nT; ++t) {
        __syncthreads();            // every wavefront is done reading the previous tile
        store_tile();
        __syncthreads();            // tile t is visible to all wavefronts
        if (t + 1 < nT) load_tile(t + 1);

        const int key0 = t * kBc;
        if (CAUSAL && key0 > wave_lim_max) continue;   // nothing visible for this wavefront's rows

        // ---- S^T = K Q^T : two 32-key blocks, fp32 accumulators
        f32x16 s[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 kf = *(const bf16x8*)(sK + k_chunk_offset<D>(qk_key_row(lane, kb), qk_chunk(lane, ks)));
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[kb], 0, 0, 0);
            }
        }

        // ---- mask: causal diagonal and keys past Sk
        if (key0 + kBc - 1 > wave_lim_min) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = key0 + 32 * kb + mfma_c_row(lane, r);
                    if (key > lim) s[kb][r] = -INFINITY;
                }
        }

        // ---- online softmax (Section 2: "accumulating into O via online softmax")
        float mx = s[0][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[0][r]);
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[1][r]);
        mx = max_across_halves(mx);
        const float m_new = fmaxf(m_run, mx);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = fast_exp2((m_run - m_use) * c);
        m_run = m_new;
        const float mc = m_use * c;
        float psum = 0.f;
        unsigned pk[2][8];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                const float p0 = fast_exp2(fmaf(s[kb][r], c, -mc));
                const float p1 = fast_exp2(fmaf(s[kb][r + 1], c, -mc));
                psum += p0 + p1;
                pk[kb][r >> 1] = pack_bf16x2(p0, p1);
            }
        l_run = l_run * alpha + psum;
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
            for (int i = 0; i < DB; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[i][r] *= alpha;
        }

        // ---- O^T += V^T P^T
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            u32x4 pw = {pk[kk >> 1][4 * (kk & 1) + 0], pk[kk >> 1][4 * (kk & 1) + 1],
                        pk[kk >> 1][4 * (kk & 1) + 2], pk[kk >> 1][4 * (kk & 1) + 3]};
            const bf16x8 pf = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
            for (int dblk = 0; dblk < DB; ++dblk) {
                const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, sV + pv_addr_offset<D>(lane, dblk, kk, 0)));
                const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, sV + pv_addr_offset<D>(lane, dblk, kk, 1)));
                typedef __attribute__((ext_vector_type(8))) short s16x8;
                const s16x8 vv = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
                oacc[dblk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vv), pf, oacc[dblk], 0, 0, 0);
            }
        }
    }

    // ---- epilogue: normalise, round once to bf16, store O and LSE
    const float l_tot = sum_across_halves(l_run);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    if (qi < Sq) {
        __bf16* orow = p.o + (((size_t)bc.b * p.Hq + bc.hq) * (size_t)Sq + qi) * D;
#pragma unroll
        for (int dblk = 0; dblk < DB; ++dblk)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                u32x2 w;
                w[0] = pack_bf16x2(oacc[dblk][4 * g4 + 0] * inv, oacc[dblk][4 * g4 + 1] * inv);
                w[1] = pack_bf16x2(oacc[dblk][4 * g4 + 2] * inv, oacc[dblk][4 * g4 + 3] * inv);
                *(u32x2*)(orow + o_d(lane, dblk, 4 * g4)) = w;
            }
        if (p.lse != nullptr && half == 0) {
            const float v = l_tot > 0.f ? m_run * p.scale + logf(l_tot) : -INFINITY;
            p.lse[((size_t)bc.b * p.Hq + bc.hq) * (size_t)Sq + qi] = v;
        }
    }
}

}  // namespace

// Host-side launcher: the only symbol the C-ABI translation unit needs from this file.
int attn_launch(const AttnParams& p, int D, int causal, hipStream_t stream) {
    const dim3 grid((unsigned)p.nblocks), block(256);
    if (D == 128) {
        if (causal) hipLaunchKernelGGL((attn_fwd_generic<128, true>), grid, block, 0, stream, p);
        else        hipLaunchKernelGGL((attn_fwd_generic<128, false>), grid, block, 0, stream, p);
    } else {
        if (causal) hipLaunchKernelGGL((attn_fwd_generic<64, true>), grid, block, 0, stream, p);
        else        hipLaunchKernelGGL((attn_fwd_generic<64, false>), grid, block, 0, stream, p);
    }
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

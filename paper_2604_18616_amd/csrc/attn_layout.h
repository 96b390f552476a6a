// Index maps of the attention-forward kernels, as plain constexpr functions that
// compile for both host and device.  The kernels use them for every LDS address
// and every MFMA lane<->element correspondence; the host tests enumerate them to
// check the operand-pairing ("tag conformity") and no-collision properties that
// the paper states as data-flow invariants ("The DSL", tag functions and assertions; the assertions at the two
// MFMA sites of Figure 1), and to count LDS bank conflicts.
//
// Tiling (cf. Figure 1: one wavefront owns 32 query rows, K/V stream through LDS
// in Bc = 64-key tiles):
//   S^T = K Q^T   per wavefront: A = K tile (32 keys x 16 d), B = Q^T (16 d x 32 queries)
//   O^T += V^T P^T per wavefront: A = V^T (32 d x 16 keys),   B = P^T (16 keys x 32 queries)
// so a lane's accumulator column is always one query row: the running max, the
// running sum and the rescale factor are per-lane scalars.
#pragma once

#if defined(__HIPCC__)
#define ATTN_HD __host__ __device__ inline
#else
#define ATTN_HD inline
#endif

namespace attn_layout {

constexpr int kBc = 64;        // keys per LDS tile
constexpr int kWaveRows = 32;  // query rows per wavefront
constexpr int kChunk = 16;     // bytes per LDS/global chunk (8 bf16)

// ---- v_mfma_f32_32x32x16_bf16 register layouts (verified on gfx950) -------------
// A operand: lane l holds A[m = l%32][k = 8*(l/32) + e], e = 0..7
// B operand: lane l holds B[k = 8*(l/32) + e][n = l%32], e = 0..7
// C/D      : lane l, register r holds C[m = 8*(r/4) + 4*(l/32) + r%4][n = l%32], r = 0..15
ATTN_HD constexpr int mfma_ab_k(int lane, int e) { return 8 * (lane / 32) + e; }
ATTN_HD constexpr int mfma_ab_mn(int lane) { return lane % 32; }
ATTN_HD constexpr int mfma_c_row(int lane, int r) { return 8 * (r / 4) + 4 * (lane / 32) + r % 4; }
ATTN_HD constexpr int mfma_c_col(int lane) { return lane % 32; }

// ---- LDS tile layout --------------------------------------------------------------
// A tile is kBc rows of D bf16 (D*2 bytes), split into D/8 chunks of 16 bytes.
// Chunk c of row r lives at chunk position (c ^ swizzle(r)) of that row.
// K is read one 16-byte chunk per lane with 32 consecutive rows per half-wave, so
// its swizzle must spread 16 consecutive rows over all 64 banks; V is read by the
// transposing 8-byte load, 4 consecutive rows x 64 contiguous bytes per half-wave,
// so its swizzle must send 4 consecutive rows to 4 different 64-byte bank groups.
template <int D> ATTN_HD constexpr int k_swizzle(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
template <int D> ATTN_HD constexpr int v_swizzle(int row) { return D == 128 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2); }
template <int D> ATTN_HD constexpr int tile_bytes() { return kBc * D * 2; }
template <int D> ATTN_HD constexpr int k_chunk_offset(int row, int chunk) { return row * (D * 2) + ((chunk ^ k_swizzle<D>(row)) * kChunk); }
template <int D> ATTN_HD constexpr int v_chunk_offset(int row, int chunk) { return row * (D * 2) + ((chunk ^ v_swizzle<D>(row)) * kChunk); }

// ---- direct HBM -> LDS copy of a tile (NW wavefronts: 8, or 4 in the 128-row workgroup) ---------
// The tile is copied by 1 KB wavefront instructions: instruction q writes LDS bytes
// [1024*q, 1024*(q+1)) lane-contiguously (lane i -> 16 bytes at 1024*q + 16*i), i.e. rows
// q*R .. q*R+R-1 with R = 1024 / (2*D) rows per instruction.  Wavefront w issues instructions
// q = w + NW*n.  The swizzle is applied on the source side: lane i fetches the global chunk
// that belongs at its fixed LDS position.  Rows of part n lie n*NW*R (a multiple of 16) below
// those of part 0, so both swizzles repeat and a lane's source offset for part n is that of
// part 0 plus the constant n*NW*R*D elements.
template <int D> ATTN_HD constexpr int dma_rows_per_inst() { return 1024 / (2 * D); }
template <int D, int NW = 8> ATTN_HD constexpr int dma_insts_per_wave() { return tile_bytes<D>() / 1024 / NW; }
template <int D, int NW = 8> ATTN_HD constexpr int dma_row(int wave, int n, int lane) { return (wave + NW * n) * dma_rows_per_inst<D>() + lane / (D / 8); }
template <int D, int NW = 8> ATTN_HD constexpr int dma_dst_offset(int wave, int n, int lane) { return (wave + NW * n) * 1024 + 16 * lane; }
// element offset within the [kBc, D] tile of the 8 bf16 that lane fetches
template <int D, bool IS_V, int NW = 8> ATTN_HD constexpr int dma_src_elem(int wave, int n, int lane) {
    const int row = dma_row<D, NW>(wave, n, lane);
    const int pos = lane % (D / 8);
    return row * D + ((pos ^ (IS_V ? v_swizzle<D>(row) : k_swizzle<D>(row))) * 8);
}

// ---- S^T = K Q^T operand fetch ------------------------------------------------------
// MFMA (kb, ks): key block kb (32 keys), reduction step ks (16 d).  Lane l reads the
// 16-byte chunk holding K[key = 32*kb + l%32][d = 16*ks + 8*(l/32) .. +7] from LDS and
// pairs it with its register copy of Q[query = l%32][same d].
ATTN_HD constexpr int qk_key_row(int lane, int kb) { return 32 * kb + lane % 32; }
ATTN_HD constexpr int qk_chunk(int lane, int ks) { return 2 * ks + lane / 32; }
ATTN_HD constexpr int qk_d(int lane, int ks, int e) { return 16 * ks + 8 * (lane / 32) + e; }

// ---- P^T as B operand of O^T += V^T P^T ---------------------------------------------
// The S^T accumulator of key block kb holds, in lane l, keys 32*kb + mfma_c_row(l, r).
// PV step kk = 2*kb + r/8 consumes registers r = 8*(kk%2) .. +7 as B-operand elements
// e = r%8, i.e. reduction slot (lane/32, e) of step kk stands for tile key
//   pv_key(lane, kk, e) = 16*kk + 8*(e/4) + 4*(lane/32) + e%4 .
ATTN_HD constexpr int pv_key(int lane, int kk, int e) { return 16 * kk + 8 * (e / 4) + 4 * (lane / 32) + e % 4; }

// ---- V^T as A operand: two transposing 8-byte LDS reads per MFMA ---------------------
// ds_read_b64_tr_b16 (verified on gfx950): lane i of a 16-lane group receives, as its
// element j, element i%4 of the 8 bytes addressed by lane 4*j + i/4 of its group.
// For MFMA (dblk, kk), read eg (0/1), lane l therefore ADDRESSES
//   row   = 16*kk + 8*eg + 4*(l/32) + (l%16)/4
//   d     = 32*dblk + 16*((l%32)/16) + 4*(l%4)          (4 consecutive d, 8 bytes)
// and RECEIVES V[key = 16*kk + 8*eg + 4*(l/32) + j][d = 32*dblk + l%32], j = 0..3,
// which is A-operand element e = 4*eg + j: the same key as pv_key(l, kk, e).
ATTN_HD constexpr int pv_addr_row(int lane, int kk, int eg) { return 16 * kk + 8 * eg + 4 * (lane / 32) + (lane % 16) / 4; }
ATTN_HD constexpr int pv_addr_d(int lane, int dblk) { return 32 * dblk + 16 * ((lane % 32) / 16) + 4 * (lane % 4); }
ATTN_HD constexpr int tr_src_lane(int lane, int j) { return (lane & ~15) + 4 * j + (lane % 16) / 4; }
ATTN_HD constexpr int tr_src_elem(int lane) { return lane % 4; }
template <int D> ATTN_HD constexpr int pv_addr_offset(int lane, int dblk, int kk, int eg) {
    return v_chunk_offset<D>(pv_addr_row(lane, kk, eg), pv_addr_d(lane, dblk) / 8) + 2 * (pv_addr_d(lane, dblk) % 8);
}

// ---- O^T accumulator -> output element ----------------------------------------------
// Accumulator dblk, register r of lane l is O[query = l%32][d = 32*dblk + mfma_c_row(l, r)].
ATTN_HD constexpr int o_d(int lane, int dblk, int r) { return 32 * dblk + mfma_c_row(lane, r); }

// ---- O staging tile of one wavefront (epilogue transpose) ------------------------------
// 32 rows x D bf16, rows of 16-byte chunks; logical chunk c of row r sits at chunk position
// c ^ (r % chunks_per_row), so the 8-byte register writes (32 rows at one d) and the 16-byte
// row reads are both conflict-free.
template <int D> ATTN_HD constexpr int o_stage_offset(int row, int d) {
    return row * (D * 2) + ((((d / 8) ^ (row % (D / 8)))) * kChunk) + 2 * (d % 8);
}
template <int D> ATTN_HD constexpr int o_stage_chunk(int row, int pos) { return pos ^ (row % (D / 8)); }

// ---- workgroup id -> block of the problem ---------------------------------------------------------
// Workgroup id -> (batch, first query head, query tile).  Workgroups are handed to the 8 XCDs
// round-robin, and each XCD has its own L2: give every XCD a contiguous range of the
// logical order, in which all query tiles of the gqa heads that share one kv head are
// neighbours, so that one XCD's resident workgroups stream the same K/V through its L2.
// Causal: heavy (late) query tiles first.
// hpw = query heads of one kv head that a workgroup covers side by side (1 for the generic kernel): its
// wavefronts then take the same row range of hpw heads instead of hpw times as many rows of one head.
struct BlockCoord { int b, hq, hk, qt; };
template <bool CAUSAL>
ATTN_HD __attribute__((always_inline)) BlockCoord block_coord(int bid, int nblocks, int Hq, int Hkv, int nQt, int hpw) {
    const int g = Hq / Hkv;
    const int gg = g / hpw;                       // head groups per kv head
    const int per_xcd = nblocks >> 3;
    const int logical = (bid < per_xcd * 8) ? (bid & 7) * per_xcd + (bid >> 3) : bid;
    const int W = gg * nQt;
    const int pair = logical / W, rem = logical - pair * W;
    int ord = rem / gg;
    const int hin = rem - ord * gg;
    // Causal tiles go heaviest first.  If one kv head's workgroups are more than an XCD's share (many query
    // heads per kv head), a heavy-first order would give one XCD the long tiles and the next the short ones:
    // then the order alternates longest, shortest, second longest, ... so that every stretch of it is balanced.
    if (CAUSAL && W > per_xcd && per_xcd > 0) ord = (ord & 1) ? nQt - 1 - (ord >> 1) : (ord >> 1);
    BlockCoord c;
    c.b = pair / Hkv;
    c.hk = pair - c.b * Hkv;
    c.hq = c.hk * g + hin * hpw;
    c.qt = CAUSAL ? nQt - 1 - ord : ord;
    return c;
}

}  // namespace attn_layout

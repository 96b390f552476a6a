// Index maps of the tiled bf16 GEMM kernel, as constexpr functions shared by the kernel and
// by the host-side layout test (which checks, for every lane and element, that both MFMA
// operands of a product carry the same k, that staging is a bijection, and how LDS banks
// are hit).  No arithmetic of the method itself lives here.
//
// The kernel computes C^T tiles: D'[n][m] += sum_k Bop[n][k] * Aop[k][m] with
// v_mfma_f32_32x32x16_bf16, whose operand / result layout for lane l is (gfx950):
//     first operand  (8 bf16): row  n = l % 32, k = 8*(l/32) + e
//     second operand (8 bf16): col  m = l % 32, k = 8*(l/32) + e
//     result (16 fp32)       : row  n = 8*(r/4) + 4*(l/32) + r%4,  col m = l % 32
// so one lane ends up with 4 consecutive n of one C row m per register quad.
#pragma once

#define GEMM_HD __host__ __device__ constexpr

namespace gemm_layout {

constexpr int kWaveN = 64;                      // every wavefront tile is 64 wide in n (C staging rows of 128 bytes)

// Workgroup tile BM x BN computed by WM x WN wavefronts, streamed in NS LDS stages of BK along k.
//   Tile<256, 256, 2, 4, 64, 2>: the large-problem shape (wavefront tile 128 x 64, one workgroup per CU);
//   Tile<256, 256, 2, 4, 32, 4>: the same tile in four half-depth stages (three copies in flight);
//   Tile<128, 128, 2, 2, 64, 2>: four times the workgroups for problems that would leave CUs idle
//                                (wavefront tile 64 x 64, two workgroups per CU);
//   Tile<128, 128, 2, 2, 64, 4>: the same tile in four stages (128 KB, one workgroup per CU, three stages of
//                                copies in flight) for problems with at most one such tile per CU;
//   Tile<64, 64, 2, 1, 64, 4>:   sixteen times the workgroups, two wavefronts of 32 x 64 each, four stages:
//                                for the smallest problems, where the time is the L2 -> LDS traffic of the
//                                busiest CU and spreading it over every CU matters more than operand reuse.
//   Tile<256, 256, 2, 4, 64, 2, 16>: the large-problem shape on v_mfma_f32_16x16x32_bf16 (MI = 16), the instruction
//                                that takes less power per FLOP on normally distributed operands;
//   Tile<192, 256, 2, 4, 64, 2, 16>: 192 rows of C (wavefront tile 96 x 64, 24 KB of A and 32 KB of B per stage) for
//                                results that 256 x 256 tiles cut into a poor number of workgroups.
template <int BM_, int BN_, int WM_, int WN_, int BK_, int NS_, int MI_ = 32>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, BK = BK_, NS = NS_, MI = MI_;
    // sub-steps per stage: MI = 32: one 16-deep reduction step over the whole wavefront tile each;
    // MI = 16: half the wavefront tile's rows (m) of one 32-deep reduction step each
    static constexpr int kKS = BK / 16;
    static constexpr int kRBK = BK * 2;                                     // bytes of a k-major tile row: 128 or 64
    static constexpr int kWaves = WM * WN;
    static constexpr int kWaveM = BM / WM;
    static constexpr int kMB = kWaveM / 32, kNB = kWaveN / 32;
    static constexpr int kStageA = BM * BK * 2, kStageB = BN * BK * 2;     // bytes of one operand, one stage
    static constexpr int kBOffset = NS * kStageA;                           // B stages follow the A stages
    static constexpr int kLdsBytes = NS * (kStageA + kStageB);
    static constexpr int kPerCU = (WM * WN == 8 || kLdsBytes > 80 * 1024) ? 1 : 2;   // workgroups meant to share a CU (160 KB of LDS)
    static constexpr int kCopiers = kWaves < 4 ? kWaves : 4;                // copying wavefronts (one per SIMD)
    static constexpr int kCopiesA = kStageA / 1024 / kCopiers, kCopiesB = kStageB / 1024 / kCopiers;   // 1 KB instructions per copier and stage
    static constexpr int kNRowBytes = BN * 2;                               // row of the [k][n] tile of B stored [K,N]
    static_assert(BN / WN == kWaveN && kWaveM % 32 == 0 && kCopiesA >= 1 && kCopiesB >= 1 && (BK == 64 || BK == 32) && kKS % 2 == 0 && NS >= 2,
                  "unsupported tile");
};
using TileLarge = Tile<256, 256, 2, 4, 64, 2>;
using TileLarge4 = Tile<256, 256, 2, 4, 32, 4>;
using TileSmall = Tile<128, 128, 2, 2, 64, 2>;
using TileTiny = Tile<64, 64, 2, 1, 64, 4>;
using TileSmall4 = Tile<128, 128, 2, 2, 64, 4>;
using TileLarge16 = Tile<256, 256, 2, 4, 64, 2, 16>;
using TileLarge4_16 = Tile<256, 256, 2, 4, 32, 4, 16>;
using TileTall16 = Tile<192, 256, 2, 4, 64, 2, 16>;      // 192 x 256: for results that 256 x 256 tiles cut into a poor number of workgroups
using TileSmall16 = Tile<128, 128, 2, 2, 64, 2, 16>;
using TileSmall4_16 = Tile<128, 128, 2, 2, 64, 4, 16>;
using TileTiny16 = Tile<64, 64, 2, 1, 64, 4, 16>;

GEMM_HD int mfma_k(int lane, int e) { return 8 * (lane >> 5) + e; }
GEMM_HD int mfma_rc(int lane) { return lane & 31; }                       // operand row (n) / col (m)
GEMM_HD int mfma_out_row(int lane, int r) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

// v_mfma_f32_16x16x32_bf16, lane l: first operand (8 bf16) row n = l % 16, k = 8*(l/16) + e; second operand col
// m = l % 16, same k; result (4 fp32) row n = 4*(l/16) + r, col m = l % 16: again 4 consecutive n of one C row m.
GEMM_HD int mfma16_k(int lane, int e) { return 8 * (lane >> 4) + e; }
GEMM_HD int mfma16_rc(int lane) { return lane & 15; }
GEMM_HD int mfma16_out_row(int lane, int r) { return 4 * (lane >> 4) + r; }

// ---- tiles whose rows run along k (A; B stored [N,K]): BM or BN rows x RBK bytes (128 or 64) --
// 16-byte chunk c of row r sits at chunk position c ^ kswz(r): 16 consecutive rows of one
// chunk column then cover all 64 banks.
template <int RBK = 128> GEMM_HD int kswz(int row) { return RBK == 128 ? (row >> 1) & 7 : (row >> 2) & 3; }
template <int RBK = 128> GEMM_HD int kt_offset(int row, int chunk) { return row * RBK + ((chunk ^ kswz<RBK>(row)) << 4); }
// operand of 32-row block `blk`, reduction step ks: one 16-byte read per lane
GEMM_HD int kt_row(int blk, int lane) { return blk * 32 + (lane & 31); }
GEMM_HD int kt_chunk(int ks, int lane) { return 2 * ks + (lane >> 5); }
// the same for the 16x16x32 instruction: 16-row block `blk`, 32-deep step ks
GEMM_HD int kt16_row(int blk, int lane) { return blk * 16 + (lane & 15); }
GEMM_HD int kt16_chunk(int ks, int lane) { return 4 * ks + (lane >> 4); }
// direct-to-LDS copy, instruction i (1024 / RBK rows each): lane's 16 bytes land at i*1024 + lane*16
template <int RBK = 128> GEMM_HD int kt_dma_row(int i, int lane) { return (1024 / RBK) * i + lane / (RBK / 16); }
template <int RBK = 128> GEMM_HD int kt_dma_chunk(int i, int lane) { return (lane % (RBK / 16)) ^ kswz<RBK>(kt_dma_row<RBK>(i, lane)); }

// ---- B stored [K,N]: tile of BK k-rows x RB bytes (RB = 2 BN: 512, 256 or 128) -----------------
// read with ds_read_b64_tr_b16: in a 16-lane group, lane i receives as element j the element
// i%4 of the 8 bytes addressed by lane 4*j + i/4.  Four consecutive k rows are XORed onto
// four different 64-byte groups of the 256-byte bank line (128-byte rows: two rows share a bank
// line, so rows k and k+2 take different halves of their row).
// MI = 16 (rows of 256 bytes and more only): the two 16-lane groups of a 32-lane access read k rows 8 apart, which
// take different 32-byte halves of their 64-byte group.
template <int RB, int MI = 32> GEMM_HD int nswz(int krow) {
    return (RB >= 256 ? (krow & 3) << 2 : ((krow >> 1) & 1) << 2) | (MI == 16 ? ((krow >> 3) & 1) << 1 : 0);
}
template <int RB, int MI = 32> GEMM_HD int nt_offset(int krow, int chunk) { return krow * RB + ((chunk ^ nswz<RB, MI>(krow)) << 4); }
// address lane `lane` supplies for read x (0,1) of n-block nb (32 columns), step ks
GEMM_HD int tr_krow(int ks, int x, int lane) { return ks * 16 + 8 * (lane >> 5) + 4 * x + ((lane & 15) >> 2); }
GEMM_HD int tr_ncol(int nb, int lane) { return nb * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3); }
template <int RB> GEMM_HD int tr_offset(int nb, int ks, int x, int lane) {
    return nt_offset<RB>(tr_krow(ks, x, lane), tr_ncol(nb, lane) >> 3) + ((tr_ncol(nb, lane) & 7) << 1);
}
// the 16x16x32 operand: n-block nb of 16 columns, 32-deep step ks; every 16-lane group covers the same 16 columns
GEMM_HD int tr16_krow(int ks, int x, int lane) { return ks * 32 + 8 * (lane >> 4) + 4 * x + ((lane & 15) >> 2); }
GEMM_HD int tr16_ncol(int nb, int lane) { return nb * 16 + 4 * (lane & 3); }
template <int RB> GEMM_HD int tr16_offset(int nb, int ks, int x, int lane) {
    return nt_offset<RB, 16>(tr16_krow(ks, x, lane), tr16_ncol(nb, lane) >> 3) + ((tr16_ncol(nb, lane) & 7) << 1);
}
// which lane's address, and which of its 4 elements, ends up as element j of lane `lane`
GEMM_HD int tr_src_lane(int lane, int j) { return (lane & ~15) + 4 * j + ((lane & 15) >> 2); }
GEMM_HD int tr_src_elem(int lane) { return lane & 3; }
// copy instruction i: 1024 / RB k rows of RB bytes
template <int RB> GEMM_HD int nt_dma_row(int i, int lane) { return (1024 / RB) * i + lane / (RB / 16); }
template <int RB, int MI = 32> GEMM_HD int nt_dma_chunk(int i, int lane) { return (lane % (RB / 16)) ^ nswz<RB, MI>(nt_dma_row<RB>(i, lane)); }

// ---- issue order of a stage's copy instructions ---------------------------------------------------
// Per copying wavefront a stage has ca parts of A (numbered 0 .. ca-1) and cb >= ca parts of B (numbered ca .. ca+cb-1).
// They are issued A part, B part in turn, then the B parts left over: position n of the order is part
GEMM_HD int copy_order(int n, int ca) { return n < 2 * ca ? ((n & 1) ? ca + n / 2 : n / 2) : n; }

// ---- C staging (epilogue): per wavefront kWaveM rows (m) x 128 bytes (64 n) ------------------
GEMM_HD int cswz(int m) { return (m >> 1) & 7; }
GEMM_HD int c_stage_offset(int m, int n) { return m * 128 + (((n >> 3) ^ cswz(m)) << 4) + ((n & 7) << 1); }

// ---- workgroup id -> C tile ------------------------------------------------------------------
// Workgroups go to the 8 XCDs round-robin and each XCD has its own L2: every XCD gets a
// contiguous range of the logical order, and the logical order walks the tiles in bands of GEMM_GM (4)
// tile rows, column by column, so that the ~32 workgroups resident on one XCD cover a 4 x 8
// patch of C and share 12 operand panels instead of 64.
struct TileCoord { int tm, tn; };
GEMM_HD TileCoord tile_coord(int bid, int nblocks, int tiles_m, int tiles_n) {
    const int per_xcd = nblocks >> 3;
    const int logical = (bid < per_xcd * 8) ? (bid & 7) * per_xcd + (bid >> 3) : bid;
#ifndef GEMM_GM
#define GEMM_GM 4
#endif
    const int GM = GEMM_GM;
    const int band = logical / (GM * tiles_n);
    const int first = band * GM;
    const int rows = (tiles_m - first) < GM ? (tiles_m - first) : GM;
    const int rem = logical - band * GM * tiles_n;
    const int tn = rem / rows;
    return TileCoord{first + (rem - tn * rows), tn};
}

}  // namespace gemm_layout

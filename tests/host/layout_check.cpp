// Host-side check of the kernels' index maps (csrc/attn_layout.h), compiled with g++ by
// tests/test_layout_host.py.  These are the paper's data-flow invariants ("The DSL", tag functions and assertions: tag
// assertions at the two MFMA sites of Figure 1; non-conformity of concurrent LDS writers)
// recast as plain enumeration over every lane, register and step:
//   1. QK^T conformity: the K element a lane fetches from LDS for MFMA (kb, ks) and the Q element
//      it pairs with carry the same reduction index d, and land in the S^T row/column the mask
//      and the softmax assume.
//   2. PV conformity: the V element delivered to A-operand slot (lane, e) of MFMA (dblk, kk) by the
//      transposing load has the key index that P^T's B-operand slot (lane, e) stands for, and the
//      d index of the O^T row the lane's accumulator register is stored to.
//   3. Staging is a bijection: no two lanes of the direct-to-LDS copy write the same LDS bytes and
//      every byte of the tile is written; the swizzled chunk position is within the row.
//   4. Bank model: the K read (16 lanes x 16 B) and the V read (32 lanes x 8 B) touch every
//      4-byte bank at most once per 256-byte LDS cycle.
//   6. The workgroup-id -> block map is a bijection onto (batch, head group, query tile), keeps an XCD on one kv
//      head at a time and orders causal tiles heaviest first.
//   5. The bug class of the paper's worked example ("Agentic Optimization Harness", the attention example: an operand read through the
//      staging layout instead of the MFMA view) is detected by check 1 when planted.
#include <cstdio>
#include <cstdlib>
#include <set>
#include <vector>
#include "../../paper_2604_18616_amd/csrc/attn_layout.h"
using namespace attn_layout;

static int failures = 0;
#define CHECK(cond, ...) do { if (!(cond)) { if (failures < 20) { printf("FAIL %s:%d: ", __FILE__, __LINE__); printf(__VA_ARGS__); printf("\n"); } ++failures; } } while (0)

// LDS image of a tile after staging: for each byte, which (row, d) element it holds.  The copy
// writes 16-byte chunks: lane-contiguous LDS destination, swizzle applied on the source side.
template <int D> struct Tile { std::vector<int> row, d; Tile() : row(tile_bytes<D>(), -1), d(tile_bytes<D>(), -1) {} };

template <int D, bool IS_V, int NW = 8> Tile<D> stage() {
    Tile<D> t;
    constexpr int NDMA = dma_insts_per_wave<D, NW>();
    static_assert(NDMA * NW * 1024 == tile_bytes<D>(), "the wavefronts' copies tile the buffer");
    std::set<int> written;
    for (int wave = 0; wave < NW; ++wave)
        for (int n = 0; n < NDMA; ++n)
            for (int lane = 0; lane < 64; ++lane) {
                const int src = dma_src_elem<D, IS_V, NW>(wave, n, lane);      // element offset in the tile
                // the kernel derives load n from load 0 plus a constant number of rows
                const int src0 = dma_src_elem<D, IS_V, NW>(wave, 0, lane);
                CHECK(src == src0 + n * NW * dma_rows_per_inst<D>() * D,
                      "load %d of wave %d lane %d is not load 0 plus a constant", n, wave, lane);
                const int row = src / D, chunk = (src % D) / 8;
                const int want_row = dma_row<D, NW>(wave, n, lane);
                CHECK(src % 8 == 0 && row == want_row && row < kBc, "bad source element %d", src);
                const int dst = dma_dst_offset<D, NW>(wave, n, lane);
                const int expect = IS_V ? v_chunk_offset<D>(row, chunk) : k_chunk_offset<D>(row, chunk);
                CHECK(dst == expect, "copy destination %d != layout offset %d (row %d chunk %d)", dst, expect, row, chunk);
                for (int b = 0; b < 16; ++b) {
                    CHECK(!written.count(dst + b), "LDS byte %d written twice", dst + b);
                    written.insert(dst + b);
                    t.row[dst + b] = row; t.d[dst + b] = chunk * 8 + b / 2;
                }
            }
    CHECK((int)written.size() == tile_bytes<D>(), "tile not fully written: %zu of %d bytes", written.size(), tile_bytes<D>());
    return t;
}

template <int D> void check_qk(bool plant_bug) {
    const Tile<D> k = stage<D, false>();
    int mism = 0;
    for (int kb = 0; kb < 2; ++kb) for (int ks = 0; ks < D / 16; ++ks) for (int lane = 0; lane < 64; ++lane) {
        int off = k_chunk_offset<D>(qk_key_row(lane, kb), qk_chunk(lane, ks));
        if (plant_bug) off = qk_key_row(lane, kb) * (D * 2) + qk_chunk(lane, ks) * 16;   // read through the unswizzled view
        for (int e = 0; e < 8; ++e) {
            const int row = k.row[off + 2 * e], d = k.d[off + 2 * e];
            const bool ok = row == 32 * kb + mfma_ab_mn(lane)                  // A-operand row m = key within the block
                         && d == qk_d(lane, ks, e)                             // same reduction index as the Q fragment
                         && qk_d(lane, ks, e) == 16 * ks + mfma_ab_k(lane, e); // which is MFMA reduction slot k
            if (!ok) ++mism;
        }
    }
    if (plant_bug) CHECK(mism > 0, "planted staging-view bug was not detected (D=%d)", D);
    else CHECK(mism == 0, "QK operand pairing broken in %d elements (D=%d)", mism, D);
}

template <int D> void check_pv() {
    const Tile<D> v = stage<D, true>();
    for (int kk = 0; kk < 4; ++kk) for (int dblk = 0; dblk < D / 32; ++dblk) for (int eg = 0; eg < 2; ++eg) {
        int addr[64];
        for (int lane = 0; lane < 64; ++lane) addr[lane] = pv_addr_offset<D>(lane, dblk, kk, eg);
        for (int lane = 0; lane < 64; ++lane) for (int j = 0; j < 4; ++j) {
            const int src = addr[tr_src_lane(lane, j)] + 2 * tr_src_elem(lane);   // what the transposing load delivers
            const int e = 4 * eg + j;
            CHECK(v.row[src] == pv_key(lane, kk, e), "PV key mismatch: lane %d kk %d e %d got key %d want %d", lane, kk, e, v.row[src], pv_key(lane, kk, e));
            CHECK(v.d[src] == 32 * dblk + mfma_ab_mn(lane), "PV d mismatch: lane %d got d %d", lane, v.d[src]);
        }
    }
    // P^T: S^T accumulator register r of key block kb feeds PV step kk = 2*kb + r/8 as element r%8
    for (int lane = 0; lane < 64; ++lane) for (int kb = 0; kb < 2; ++kb) for (int r = 0; r < 16; ++r)
        CHECK(32 * kb + mfma_c_row(lane, r) == pv_key(lane, 2 * kb + r / 8, r % 8), "P/S key map broken lane %d kb %d r %d", lane, kb, r);
    // O^T accumulator rows cover each d exactly once per query column, 4 consecutive d per register group
    for (int lane = 0; lane < 64; ++lane) for (int dblk = 0; dblk < D / 32; ++dblk) for (int g4 = 0; g4 < 4; ++g4)
        for (int j = 0; j < 4; ++j) CHECK(o_d(lane, dblk, 4 * g4 + j) == o_d(lane, dblk, 4 * g4) + j, "O store group not contiguous");
    std::set<int> seen;
    for (int half = 0; half < 2; ++half) for (int dblk = 0; dblk < D / 32; ++dblk) for (int r = 0; r < 16; ++r) seen.insert(o_d(32 * half, dblk, r));
    CHECK((int)seen.size() == D, "O rows of the two half-wave lanes cover %zu of %d d", seen.size(), D);
}

// 64 banks x 4 bytes = 256 bytes per LDS cycle
template <int D> void check_banks() {
    for (int kb = 0; kb < 2; ++kb) for (int ks = 0; ks < D / 16; ++ks) for (int grp = 0; grp < 4; ++grp) {
        std::set<int> banks;
        for (int lane = 16 * grp; lane < 16 * grp + 16; ++lane) {
            const int off = k_chunk_offset<D>(qk_key_row(lane, kb), qk_chunk(lane, ks));
            for (int b = 0; b < 16; b += 4) { CHECK(!banks.count((off + b) / 4 % 64), "K read bank conflict (D=%d kb %d ks %d lane %d)", D, kb, ks, lane); banks.insert((off + b) / 4 % 64); }
        }
    }
    for (int kk = 0; kk < 4; ++kk) for (int dblk = 0; dblk < D / 32; ++dblk) for (int eg = 0; eg < 2; ++eg) for (int half = 0; half < 2; ++half) {
        std::set<int> banks;
        for (int lane = 32 * half; lane < 32 * half + 32; ++lane) {
            const int off = pv_addr_offset<D>(lane, dblk, kk, eg);
            for (int b = 0; b < 8; b += 4) { CHECK(!banks.count((off + b) / 4 % 64), "V read bank conflict (D=%d kk %d dblk %d lane %d)", D, kk, dblk, lane); banks.insert((off + b) / 4 % 64); }
        }
    }
}

// O staging tile: every (row, d) has its own bytes; the row reads recover whole rows.
template <int D> void check_o_stage() {
    std::vector<int> owner(32 * D * 2, -1);
    for (int lane = 0; lane < 64; ++lane) for (int dblk = 0; dblk < D / 32; ++dblk) for (int g4 = 0; g4 < 4; ++g4) {
        const int row = lane % 32, d0 = o_d(lane, dblk, 4 * g4);
        const int off = o_stage_offset<D>(row, d0);
        CHECK(off % 8 == 0 && off + 8 <= 32 * D * 2, "stage offset out of range");
        for (int b = 0; b < 8; ++b) { CHECK(owner[off + b] < 0, "O stage byte written twice"); owner[off + b] = row * D + d0 + b / 2; }
    }
    constexpr int CPR = D / 8;
    for (int j = 0; j < 32 / (64 / CPR); ++j) for (int lane = 0; lane < 64; ++lane) {
        const int r = j * (64 / CPR) + lane / CPR, pos = lane % CPR;
        const int d = o_stage_chunk<D>(r, pos) * 8;
        for (int b = 0; b < 16; ++b) CHECK(owner[r * D * 2 + pos * 16 + b] == r * D + d + b / 2, "O stage read/write mismatch row %d pos %d", r, pos);
    }
    // bank model: the 8-byte writes of a half-wave (32 lanes = 32 rows at one d, same half) spread over 64 banks
    for (int dblk = 0; dblk < D / 32; ++dblk) for (int g4 = 0; g4 < 4; ++g4) for (int half = 0; half < 2; ++half) {
        std::set<int> banks;
        for (int lane = 32 * half; lane < 32 * half + 32; ++lane) {
            const int off = o_stage_offset<D>(lane % 32, o_d(lane, dblk, 4 * g4));
            banks.insert(off / 4 % 64); banks.insert((off + 4) / 4 % 64);
        }
        CHECK((int)banks.size() >= (D == 128 ? 32 : 16), "O stage writes concentrate on %zu banks", banks.size());   // at most 2-way (D=128) / 4-way (D=64) conflicts; runs once per workgroup
    }
}

// The 128-row workgroup copies the same tiles with four wavefronts: same LDS image, every byte once.
template <int D> void check_four_wave_copy() {
    const Tile<D> k8 = stage<D, false, 8>(), k4 = stage<D, false, 4>(), v8 = stage<D, true, 8>(), v4 = stage<D, true, 4>();
    CHECK(k8.row == k4.row && k8.d == k4.d, "K tile image differs between the 8- and the 4-wavefront copy (D=%d)", D);
    CHECK(v8.row == v4.row && v8.d == v4.d, "V tile image differs between the 8- and the 4-wavefront copy (D=%d)", D);
}

// Workgroup id -> block: every (batch, head group, query tile) of the problem is taken by exactly one workgroup, the
// kv head is the one the query heads read, every XCD (workgroup id % 8) gets a contiguous stretch of the logical order
// in which the head groups and query tiles of one kv head are neighbours, and causal tiles come heaviest first within
// a kv head (or alternate longest / shortest when one kv head's blocks exceed an XCD's share).
template <bool CAUSAL> void check_block_coord(int B, int Hq, int Hkv, int nQt, int hpw) {
    const int g = Hq / Hkv, gg = g / hpw, nblocks = B * (Hq / hpw) * nQt;
    std::set<long long> seen;
    std::vector<int> prev_qt(8, -1), prev_pair(8, -1);
    for (int bid = 0; bid < nblocks; ++bid) {
        const BlockCoord c = block_coord<CAUSAL>(bid, nblocks, Hq, Hkv, nQt, hpw);
        CHECK(c.b >= 0 && c.b < B && c.hk >= 0 && c.hk < Hkv && c.qt >= 0 && c.qt < nQt, "block %d out of range (b %d hk %d qt %d)", bid, c.b, c.hk, c.qt);
        CHECK(c.hq % hpw == 0 && c.hq / g == c.hk && c.hq + hpw <= Hq, "block %d: heads %d..%d do not read kv head %d", bid, c.hq, c.hq + hpw - 1, c.hk);
        const long long key = ((long long)c.b * Hq + c.hq) * nQt + c.qt;
        CHECK(!seen.count(key), "block (b %d, hq %d, qt %d) taken twice", c.b, c.hq, c.qt);
        seen.insert(key);
        // within an XCD's share (full shares only), consecutive workgroups stay on a kv head until it is exhausted
        const int per_xcd = nblocks >> 3, x = bid & 7;
        if (bid < per_xcd * 8) {
            const int pair = c.b * Hkv + c.hk;
            CHECK(pair >= prev_pair[x], "XCD %d goes back from (b, hk) pair %d to %d", x, prev_pair[x], pair);
            if (CAUSAL && pair == prev_pair[x] && gg * nQt <= per_xcd) CHECK(c.qt <= prev_qt[x], "XCD %d: causal tile %d after %d is not heaviest first", x, c.qt, prev_qt[x]);
            prev_pair[x] = pair; prev_qt[x] = c.qt;
        }
    }
    CHECK((int)seen.size() == nblocks, "%zu of %d blocks covered", seen.size(), nblocks);
}

int main() {
    for (int hpw : {1, 2, 4, 8}) {
        check_block_coord<true>(4, 32, 8, 64, hpw <= 4 ? hpw : 4);                             // the headline shape and its packings
        check_block_coord<false>(2, 16, 16, 32, 1);
        check_block_coord<true>(16, 8, 1, 32, hpw);                                            // 8 query heads on one kv head
        check_block_coord<true>(1, 32, 1, 33, hpw);                                            // one kv head larger than an XCD's share, odd tile count
        check_block_coord<false>(3, 6, 2, 5, 1);                                               // not a multiple of 8 workgroups
        check_block_coord<true>(1, 2, 2, 1, 1);                                                // fewer than 8 workgroups
    }
    check_four_wave_copy<128>(); check_four_wave_copy<64>();
    check_o_stage<128>(); check_o_stage<64>();
    check_qk<128>(false); check_qk<64>(false);
    check_qk<128>(true);  check_qk<64>(true);
    check_pv<128>(); check_pv<64>();
    check_banks<128>(); check_banks<64>();
    // MFMA C layout is a bijection lane x reg -> 32 x 32
    std::set<int> cells;
    for (int lane = 0; lane < 64; ++lane) for (int r = 0; r < 16; ++r) cells.insert(mfma_c_row(lane, r) * 32 + mfma_c_col(lane));
    CHECK(cells.size() == 1024, "C layout not a bijection");
    if (failures) { printf("%d layout check(s) failed\n", failures); return 1; }
    printf("layout checks passed\n");
    return 0;
}

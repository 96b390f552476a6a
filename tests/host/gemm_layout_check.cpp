// Host-side check of the GEMM kernel's index maps (csrc/gemm_layout.h), compiled with g++ by
// tests/test_layout_host.py.  The paper's data-flow invariant for GEMM (Introduction: the MFMA
// instructions always receive correctly paired elements of A and B whatever the tiling,
// staging and swizzling in between) recast as plain enumeration over every lane and element:
//   1. staging is a bijection onto the LDS tile and the copy's lane-contiguous destination
//      equals the swizzled layout offset of the piece each lane fetches;
//   2. operand conformity: the element a lane receives for slot e of sub-step ks carries the
//      k that the MFMA contracts at that slot, and the row (n) / column (m) of the accumulator
//      it feeds; for B stored [K,N] this goes through the model of ds_read_b64_tr_b16;
//   3. bank model: 16 lanes of a 16-byte read, and 32 lanes of an 8-byte transposing read, touch
//      each 4-byte bank at most once per 256-byte LDS line;
//   4. the C staging tile: write offsets are distinct, inside the wavefront's region, and the
//      read-back map returns every (m, n) exactly once;
//   5. workgroup id -> tile is a bijection for even and ragged tile grids;
//   6. a planted swizzle mismatch between copy and operand read is detected by check 2.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <set>
#include <vector>
#define __host__
#define __device__
#include "../../paper_2604_18616_amd/csrc/gemm_layout.h"
using namespace gemm_layout;

static int failures = 0;
#define CHECK(cond, ...) do { if (!(cond)) { if (failures < 20) { printf("FAIL %s:%d: ", __FILE__, __LINE__); printf(__VA_ARGS__); printf("\n"); } ++failures; } } while (0)

struct Img { std::vector<int> row, col; explicit Img(int bytes) : row(bytes, -1), col(bytes, -1) {} };

// k-major tile (A, or B stored [N,K]): row = m or n, col = k within the stage
template <class T> static Img stage_kt() {
    constexpr int kStageBytes = T::kStageA, kBM = T::BM;
    Img t(kStageBytes);
    int written = 0;
    constexpr int RBK = T::kRBK;
    for (int i = 0; i < kStageBytes / 1024; ++i)
        for (int lane = 0; lane < 64; ++lane) {
            const int row = kt_dma_row<RBK>(i, lane), chunk = kt_dma_chunk<RBK>(i, lane);
            CHECK(row >= 0 && row < kBM && chunk >= 0 && chunk < RBK / 16, "bad source piece row %d chunk %d", row, chunk);
            const int dst = i * 1024 + lane * 16;
            const int want = kt_offset<RBK>(row, chunk);
            CHECK(dst == want, "copy destination %d != layout offset %d", dst, want);
            for (int b = 0; b < 16; ++b) {
                CHECK(t.row[dst + b] < 0, "LDS byte %d written twice", dst + b);
                t.row[dst + b] = row; t.col[dst + b] = chunk * 8 + b / 2; ++written;
            }
        }
    CHECK(written == kStageBytes, "k-major tile not fully written: %d", written);
    // the kernel's per-wavefront instruction split: copier wavefront w issues i = w + kCopiers n, every i once,
    // and its LDS destination is (w * 1024) + the assembly-time constant n * kCopiers * 1024
    std::set<int> seen;
    for (int w = 0; w < T::kCopiers; ++w) for (int n = 0; n < T::kCopiesA; ++n) seen.insert(w + T::kCopiers * n);
    CHECK((int)seen.size() == kStageBytes / 1024 && *seen.rbegin() == kStageBytes / 1024 - 1, "copy instructions not covered once");
    // the issue order of a stage's copies visits every part of A and of B exactly once
    CHECK(T::kCopiesA <= T::kCopiesB, "the copy order assumes at least as many B parts as A parts");
    std::set<int> parts;
    for (int n = 0; n < T::kCopiesA + T::kCopiesB; ++n) {
        const int j = copy_order(n, T::kCopiesA);
        CHECK(j >= 0 && j < T::kCopiesA + T::kCopiesB, "copy order position %d names part %d", n, j);
        parts.insert(j);
    }
    CHECK((int)parts.size() == T::kCopiesA + T::kCopiesB, "copy order covers %zu of %d parts", parts.size(), T::kCopiesA + T::kCopiesB);
    CHECK(T::kPerCU * (T::kLdsBytes + 256) <= 160 * 1024, "LDS budget");
    CHECK(T::kWaves * T::kWaveM * 128 <= T::kLdsBytes, "C staging does not fit the stage buffers");
    return t;
}

// n-major tile (B stored [K,N]): row = k within the stage, col = n within the tile
template <class T> static Img stage_nt() {
    constexpr int kStageBytes = T::kStageB, RB = T::kNRowBytes;
    Img t(kStageBytes);
    int written = 0;
    for (int i = 0; i < kStageBytes / 1024; ++i)
        for (int lane = 0; lane < 64; ++lane) {
            const int row = nt_dma_row<RB>(i, lane), chunk = nt_dma_chunk<RB, T::MI>(i, lane);
            CHECK(row >= 0 && row < T::BK && chunk >= 0 && chunk < RB / 16, "bad source piece row %d chunk %d", row, chunk);
            const int dst = i * 1024 + lane * 16;
            CHECK(dst == (nt_offset<RB, T::MI>(row, chunk)), "copy destination %d != layout offset %d", dst, nt_offset<RB, T::MI>(row, chunk));
            for (int b = 0; b < 16; ++b) {
                CHECK(t.row[dst + b] < 0, "LDS byte %d written twice", dst + b);
                t.row[dst + b] = row; t.col[dst + b] = chunk * 8 + b / 2; ++written;
            }
        }
    CHECK(written == kStageBytes, "n-major tile not fully written: %d", written);
    return t;
}

template <class T> static int check_kt_operand(bool plant_bug) {
    constexpr int kStageBytes = T::kStageA, kBM = T::BM;
    constexpr int RBK = T::kRBK, kKS = T::kKS;
    const Img t = stage_kt<T>();
    int mism = 0;
    for (int blk = 0; blk < kBM / 32; ++blk)
        for (int ks = 0; ks < kKS; ++ks)
            for (int lane = 0; lane < 64; ++lane) {
                const int row = kt_row(blk, lane), chunk = kt_chunk(ks, lane);
                // planted bug: the read forgets the swizzle (reads through the unswizzled view)
                const int off = plant_bug ? row * RBK + chunk * 16 : kt_offset<RBK>(row, chunk);
                if (off < 0 || off + 16 > kStageBytes) { ++mism; continue; }
                for (int e = 0; e < 8; ++e) {
                    const bool ok = t.row[off + 2 * e] == blk * 32 + mfma_rc(lane) && t.col[off + 2 * e] == ks * 16 + mfma_k(lane, e);
                    if (!ok) ++mism;
                }
            }
    return mism;
}

template <class T> static void check_kt_addressing() {
    constexpr int kStageBytes = T::kStageA > T::kStageB ? T::kStageA : T::kStageB, kBM = T::BM;
    // the kernel keeps one address per sub-step and adds block / stage offsets as immediates
    constexpr int RBK = T::kRBK, kKS = T::kKS;
    for (int blk = 0; blk < kBM / 32; ++blk)
        for (int ks = 0; ks < kKS; ++ks)
            for (int lane = 0; lane < 64; ++lane) {
                const int base = kt_offset<RBK>(kt_row(0, lane), kt_chunk(ks, lane));
                CHECK(kt_offset<RBK>(kt_row(blk, lane), kt_chunk(ks, lane)) == base + blk * 32 * RBK, "block offset is not additive");
            }
    CHECK((T::NS - 1) * kStageBytes + (T::kMB - 1) * 32 * RBK < 65536, "immediate offset of a 16-byte read exceeds 16 bits");
    CHECK((T::NS - 1) * kStageBytes + (kKS - 1) * 16 * T::kNRowBytes < 65536, "immediate offset of a transposing read exceeds 16 bits");
}

template <class T> static void check_nt_operand() {
    constexpr int kStageBytes = T::kStageB, RB = T::kNRowBytes, kBN = T::BN;
    constexpr int kKS = T::kKS;
    const Img t = stage_nt<T>();
    for (int nb = 0; nb < kBN / 32; ++nb)
        for (int ks = 0; ks < kKS; ++ks)
            for (int lane = 0; lane < 64; ++lane)
                for (int x = 0; x < 2; ++x) {
                    CHECK(tr_offset<RB>(nb, ks, x, lane) == tr_offset<RB>(nb, 0, x, lane) + ks * 16 * RB, "sub-step offset is not additive");
                    for (int j = 0; j < 4; ++j) {
                        const int s = tr_src_lane(lane, j);
                        const int off = tr_offset<RB>(nb, ks, x, s) + 2 * tr_src_elem(lane);
                        CHECK(off >= 0 && off + 2 <= kStageBytes && (tr_offset<RB>(nb, ks, x, s) & 7) == 0, "bad transposing-read address %d", off);
                        const int e = 4 * x + j;
                        CHECK(t.row[off] == ks * 16 + mfma_k(lane, e), "k mismatch nb %d ks %d lane %d e %d: %d", nb, ks, lane, e, t.row[off]);
                        CHECK(t.col[off] == nb * 32 + mfma_rc(lane), "n mismatch nb %d lane %d e %d: %d", nb, lane, e, t.col[off]);
                    }
                }
}

template <class T> static void check_banks() {
    constexpr int RB = T::kNRowBytes, kBM = T::BM, kBN = T::BN, RBK = T::kRBK, kKS = T::kKS;
    for (int blk = 0; blk < kBM / 32; ++blk)
        for (int ks = 0; ks < kKS; ++ks)
            for (int g = 0; g < 4; ++g) {                       // 16 lanes x 16 bytes = one 256-byte line
                std::set<int> slots;
                for (int l = 16 * g; l < 16 * g + 16; ++l) slots.insert((kt_offset<RBK>(kt_row(blk, l), kt_chunk(ks, l)) >> 4) & 15);
                CHECK(slots.size() == 16, "16-byte read: bank conflict in lane group %d (blk %d ks %d)", g, blk, ks);
            }
    for (int nb = 0; nb < kBN / 32; ++nb)
        for (int ks = 0; ks < kKS; ++ks)
            for (int x = 0; x < 2; ++x)
                for (int h = 0; h < 2; ++h) {                   // 32 lanes x 8 bytes = one 256-byte line
                    std::set<int> slots;
                    for (int l = 32 * h; l < 32 * h + 32; ++l) slots.insert((tr_offset<RB>(nb, ks, x, l) >> 3) & 31);
                    CHECK(slots.size() == 32, "transposing read: bank conflict (nb %d ks %d x %d half %d)", nb, ks, x, h);
                }
}

template <class T> static void check_c_stage() {
    constexpr int kWaveM = T::kWaveM, kNB = T::kNB, kMB = T::kMB;
    std::vector<int> m_of(kWaveM * 128, -1), n_of(kWaveM * 128, -1);
    for (int lane = 0; lane < 64; ++lane)
        for (int in = 0; in < kNB; ++in)
            for (int jm = 0; jm < kMB; ++jm)
                for (int r = 0; r < 16; ++r) {
                    const int m = jm * 32 + mfma_rc(lane), n = in * 32 + mfma_out_row(lane, r);
                    const int off = c_stage_offset(m, n);
                    CHECK(off >= 0 && off + 2 <= kWaveM * 128, "C staging offset %d out of the wavefront's region", off);
                    CHECK(m_of[off] < 0, "C staging byte %d written twice", off);
                    m_of[off] = m; n_of[off] = n; m_of[off + 1] = m; n_of[off + 1] = n;
                    // a register quad must be 8 contiguous, 8-byte aligned bytes
                    if ((r & 3) == 0) CHECK((off & 7) == 0 && c_stage_offset(m, n + 3) == off + 6, "quad not contiguous");
                }
    std::set<long> seen;
    for (int it = 0; it < kWaveM / 8; ++it)
        for (int lane = 0; lane < 64; ++lane) {
            const int row = it * 8 + (lane >> 3), pos = lane & 7, col = 8 * (pos ^ cswz(row));
            for (int e = 0; e < 8; ++e) {
                const int off = row * 128 + pos * 16 + 2 * e;
                CHECK(m_of[off] == row && n_of[off] == col + e, "read-back (%d,%d) finds (%d,%d)", row, col + e, m_of[off], n_of[off]);
                seen.insert((long)row * 64 + col + e);
            }
        }
    CHECK(seen.size() == (size_t)kWaveM * kWaveN, "read-back covers %zu of %d outputs", seen.size(), kWaveM * kWaveN);
    // write banks: 32 lanes x 8 bytes of one register quad
    for (int g = 0; g < 4; ++g)
        for (int h = 0; h < 2; ++h) {
            std::vector<int> hits(32, 0);
            int worst = 0;
            for (int l = 32 * h; l < 32 * h + 32; ++l) {
                const int off = c_stage_offset(mfma_rc(l), 8 * g + 4 * h);
                worst = std::max(worst, ++hits[(off >> 3) & 31]);
            }
            CHECK(worst <= 2, "C staging write: %d-way bank conflict", worst);
        }
}

static void check_tile_coord() {
    const int grids[][2] = {{1, 1}, {4, 4}, {32, 32}, {3, 5}, {9, 7}, {64, 64}, {17, 1}, {1, 23}, {11, 16}};
    for (auto& g : grids) {
        const int tm = g[0], tn = g[1], nb = tm * tn;
        std::set<int> seen;
        for (int bid = 0; bid < nb; ++bid) {
            const TileCoord c = tile_coord(bid, nb, tm, tn);
            CHECK(c.tm >= 0 && c.tm < tm && c.tn >= 0 && c.tn < tn, "tile (%d,%d) outside %dx%d grid", c.tm, c.tn, tm, tn);
            seen.insert(c.tm * tn + c.tn);
        }
        CHECK((int)seen.size() == nb, "%dx%d grid: %zu distinct tiles of %d", tm, tn, seen.size(), nb);
    }
}

// ---- the same checks for the 16x16x32 instruction (Tile::MI == 16) ----------------------------
template <class T> static void check_mi16() {
    constexpr int RBK = T::kRBK, RB = T::kNRowBytes, kK32 = T::BK / 32;
    const Img kt = stage_kt<T>();
    int mism = 0, planted = 0;
    for (int blk = 0; blk < T::BM / 16; ++blk)
        for (int ks = 0; ks < kK32; ++ks)
            for (int lane = 0; lane < 64; ++lane) {
                const int row = kt16_row(blk, lane), chunk = kt16_chunk(ks, lane);
                const int off = kt_offset<RBK>(row, chunk), off_bug = row * RBK + chunk * 16;
                CHECK(off == kt_offset<RBK>(kt16_row(0, lane), kt16_chunk(ks, lane)) + blk * 16 * RBK, "block offset is not additive");
                for (int e = 0; e < 8; ++e) {
                    if (!(kt.row[off + 2 * e] == blk * 16 + mfma16_rc(lane) && kt.col[off + 2 * e] == ks * 32 + mfma16_k(lane, e))) ++mism;
                    if (!(kt.row[off_bug + 2 * e] == blk * 16 + mfma16_rc(lane) && kt.col[off_bug + 2 * e] == ks * 32 + mfma16_k(lane, e))) ++planted;
                }
            }
    CHECK(mism == 0, "16x16x32: k-major operand read does not conform (%d)", mism);
    CHECK(planted > 0, "16x16x32: planted swizzle bug was not detected");
    CHECK((T::NS - 1) * T::kStageA + (T::BM / T::WM / 16 - 1) * 16 * RBK < 65536, "immediate offset of a 16-byte read exceeds 16 bits");
    const Img nt = stage_nt<T>();
    for (int nb = 0; nb < T::BN / 16; ++nb)
        for (int ks = 0; ks < kK32; ++ks)
            for (int lane = 0; lane < 64; ++lane)
                for (int x = 0; x < 2; ++x) {
                    CHECK(tr16_offset<RB>(nb, ks, x, lane) == tr16_offset<RB>(nb, 0, x, lane) + ks * 32 * RB, "32-deep step offset is not additive");
                    for (int j = 0; j < 4; ++j) {
                        const int src = tr_src_lane(lane, j);
                        const int base = tr16_offset<RB>(nb, ks, x, src);
                        const int off = base + 2 * tr_src_elem(lane);
                        CHECK(off >= 0 && off + 2 <= T::kStageB && (base & 7) == 0, "bad transposing-read address %d", off);
                        const int e = 4 * x + j;
                        CHECK(nt.row[off] == ks * 32 + mfma16_k(lane, e), "16x16x32 k mismatch nb %d ks %d lane %d e %d: %d", nb, ks, lane, e, nt.row[off]);
                        CHECK(nt.col[off] == nb * 16 + mfma16_rc(lane), "16x16x32 n mismatch nb %d lane %d e %d: %d", nb, lane, e, nt.col[off]);
                    }
                }
    CHECK((T::NS - 1) * T::kStageB + (kK32 - 1) * 32 * RB < 65536, "immediate offset of a transposing read exceeds 16 bits");
    // banks
    for (int blk = 0; blk < T::BM / 16; ++blk)
        for (int ks = 0; ks < kK32; ++ks)
            for (int g = 0; g < 4; ++g) {
                std::set<int> slots;
                for (int l = 16 * g; l < 16 * g + 16; ++l) slots.insert((kt_offset<RBK>(kt16_row(blk, l), kt16_chunk(ks, l)) >> 4) & 15);
                CHECK(slots.size() == 16, "16x16x32 16-byte read: bank conflict in lane group %d (blk %d ks %d)", g, blk, ks);
            }
    for (int nb = 0; nb < T::BN / 16; ++nb)
        for (int ks = 0; ks < kK32; ++ks)
            for (int x = 0; x < 2; ++x)
                for (int h = 0; h < 2; ++h) {
                    std::set<int> slots;
                    for (int l = 32 * h; l < 32 * h + 32; ++l) slots.insert((tr16_offset<RB>(nb, ks, x, l) >> 3) & 31);
                    CHECK(slots.size() == 32, "16x16x32 transposing read: bank conflict (nb %d ks %d x %d half %d)", nb, ks, x, h);
                }
    // C staging: 16 x 16 result blocks, a lane's 4 registers are 4 consecutive n of row m
    constexpr int kWaveM = T::kWaveM;
    std::vector<int> m_of(kWaveM * 128, -1), n_of(kWaveM * 128, -1);
    for (int lane = 0; lane < 64; ++lane)
        for (int in = 0; in < kWaveN / 16; ++in)
            for (int jm = 0; jm < kWaveM / 16; ++jm)
                for (int r = 0; r < 4; ++r) {
                    const int m = jm * 16 + mfma16_rc(lane), n = in * 16 + mfma16_out_row(lane, r);
                    const int off = c_stage_offset(m, n);
                    CHECK(off >= 0 && off + 2 <= kWaveM * 128 && m_of[off] < 0, "16x16x32 C staging byte %d bad or written twice", off);
                    m_of[off] = m; n_of[off] = n; m_of[off + 1] = m; n_of[off + 1] = n;
                    if (r == 0) CHECK((off & 7) == 0 && c_stage_offset(m, n + 3) == off + 6, "quad not contiguous");
                }
    for (int it = 0; it < kWaveM / 8; ++it)
        for (int lane = 0; lane < 64; ++lane) {
            const int row = it * 8 + (lane >> 3), pos = lane & 7, col = 8 * (pos ^ cswz(row));
            for (int e = 0; e < 8; ++e) {
                const int off = row * 128 + pos * 16 + 2 * e;
                CHECK(m_of[off] == row && n_of[off] == col + e, "16x16x32 read-back (%d,%d) finds (%d,%d)", row, col + e, m_of[off], n_of[off]);
            }
        }
    for (int h = 0; h < 2; ++h) {                                  // write banks: 32 lanes x 8 bytes
        std::vector<int> hits(32, 0);
        int worst = 0;
        for (int l = 32 * h; l < 32 * h + 32; ++l) worst = std::max(worst, ++hits[(c_stage_offset(mfma16_rc(l), mfma16_out_row(l, 0)) >> 3) & 31]);
        CHECK(worst <= 1, "16x16x32 C staging write: %d lanes on one bank pair", worst);
    }
}

template <class T> static void check_tile_shape() {
    if constexpr (T::MI == 16) { check_mi16<T>(); return; }
    CHECK(check_kt_operand<T>(false) == 0, "k-major operand read does not conform");
    CHECK(check_kt_operand<T>(true) > 0, "planted swizzle bug was not detected");
    check_kt_addressing<T>();
    check_nt_operand<T>();
    check_banks<T>();
    check_c_stage<T>();
}

int main() {
    check_tile_shape<TileLarge>();
    check_tile_shape<TileLarge4>();
    check_tile_shape<TileSmall>();
    check_tile_shape<TileTiny>();
    check_tile_shape<TileSmall4>();
    check_tile_shape<TileLarge16>();
    check_tile_shape<TileTall16>();
    check_tile_shape<TileLarge4_16>();
    check_tile_shape<TileSmall16>();
    check_tile_shape<TileSmall4_16>();
    check_tile_shape<TileTiny16>();
    check_tile_coord();
    if (failures) { printf("%d gemm layout check(s) FAILED\n", failures); return 1; }
    printf("gemm layout checks passed\n");
    return 0;
}

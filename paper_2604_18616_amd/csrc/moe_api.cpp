// C ABI of the fused MoE feed-forward: argument validation, workspace carve-up, dispatch.
// Every check runs before the first HIP call.  See include/moe.h for the contract.
#include <stdint.h>

#include "../../include/attn.h"
#include "../../include/moe.h"
#include "moe_launch.h"

static_assert(kMoeStaticScratchBytes == MOE_FFN_FP8_STATIC_MAX_BYTES, "moe.h states the size of the library-owned scratch array");

static bool sizes_ok(int T, int H, int I, int E, int KTOP) {
    if (T <= 0 || H <= 0 || I <= 0 || E <= 0 || KTOP <= 0) return false;
    if (H % 128 || I % 128 || H > 16384 || I > 16384) return false;
    if (E > 256 || KTOP > 16) return false;
    if ((long long)T * KTOP > (1LL << 20)) return false;
    // 32-bit byte offsets of the tile copies: every activation matrix stays under 4 GiB
    if ((long long)T * H >= (1LL << 32) || (long long)T * KTOP * I >= (1LL << 32)) return false;
    return true;
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

size_t moe_workspace_layout(int T, int H, int I, int E, int KTOP, size_t off[13]) {
    const size_t slots = (size_t)T * KTOP, max_tiles = (slots + kMoeBM - 1) / kMoeBM + E;
    size_t cur = 0;
    auto take = [&](int idx, size_t bytes) { off[idx] = cur; cur = align256(cur + bytes); };
    take(0, sizeof(int) * (E + 1));          // offsets
    take(1, sizeof(int) * E);                // cursor
    take(2, sizeof(int));                    // ntiles
    take(3, 4 * sizeof(int) * max_tiles);    // tile_rec
    take(4, sizeof(int));                    // (not in use)
    take(5, sizeof(int));                    // (not in use)
    take(6, sizeof(int) * slots);            // sorted_tok
    take(7, sizeof(int) * slots);            // pos
    take(8, (size_t)T * H);                  // xq
    take(9, sizeof(float) * (size_t)T * (H / 128));   // xs
    take(10, slots * I);                     // aq
    take(11, sizeof(float) * slots * (I / 128));      // as
    take(12, sizeof(float) * slots * H);     // o
    return cur;
}

extern "C" size_t moe_ffn_fp8_workspace_bytes(int T, int H, int I, int E, int KTOP) {
    if (!sizes_ok(T, H, I, E, KTOP)) return 0;
    size_t off[13];
    return moe_workspace_layout(T, H, I, E, KTOP, off);
}

extern "C" long long moe_ffn_fp8_workspace_offset(int T, int H, int I, int E, int KTOP, int part) {
    if (!sizes_ok(T, H, I, E, KTOP) || part < 0 || part > 12) return -1;
    size_t off[13];
    moe_workspace_layout(T, H, I, E, KTOP, off);
    return (long long)off[part];
}

extern "C" int moe_ffn_fp8_ex(const void* x, const int* ids, const float* wts,
                              const void* w13, const float* s13, const void* w2, const float* s2,
                              void* y, int T, int H, int I, int E, int KTOP,
                              void* workspace, size_t workspace_bytes,
                              int first_stage, int last_stage, int row_tile, void* stream) {
    if (first_stage < 0 || last_stage > 4 || first_stage > last_stage) return ATTN_ERR_UNSUPPORTED;
    if (row_tile != 0 && row_tile != 64 && row_tile != 128) return ATTN_ERR_UNSUPPORTED;
    const int bm_override = row_tile;
    if (!x || !ids || !wts || !w13 || !s13 || !w2 || !s2 || !y || !workspace) return ATTN_ERR_NULL_PTR;
    if (!sizes_ok(T, H, I, E, KTOP)) return ATTN_ERR_BAD_SHAPE;
    size_t off[13];
    const size_t need = moe_workspace_layout(T, H, I, E, KTOP, off);
    if (workspace_bytes < need) return ATTN_ERR_BAD_SHAPE;
    if (((uintptr_t)x | (uintptr_t)w13 | (uintptr_t)w2 | (uintptr_t)y) & 15u) return ATTN_ERR_MISALIGNED;
    if ((uintptr_t)workspace & 255u) return ATTN_ERR_MISALIGNED;
    if (((uintptr_t)ids | (uintptr_t)wts | (uintptr_t)s13 | (uintptr_t)s2) & 3u) return ATTN_ERR_MISALIGNED;

    char* ws = (char*)workspace;
    MoeParams p;
    p.x = (const __bf16*)x; p.ids = ids; p.wts = wts;
    p.w13 = (const uint8_t*)w13; p.s13 = s13; p.w2 = (const uint8_t*)w2; p.s2 = s2;
    p.y = (__bf16*)y;
    p.T = T; p.H = H; p.I = I; p.E = E; p.KTOP = KTOP;
    // rows of one expert per row tile: 128 (a remainder of up to 32 rows joins the tile before it, and each tile
    // runs the 64-, 128- or 160-row code that fits the rows it really has); `bm_override` is for tests
    p.bm = bm_override ? bm_override : 128;
    p.max_tiles = (int)(((size_t)T * KTOP + p.bm - 1) / p.bm + E);
    // narrow column tiles of the down product are for problems whose wide tiles would not fill the chip: the grid is
    // sized for them only if the upper bound on the row tiles is small enough for that to be possible
    p.dn_narrow_ok = (long long)p.max_tiles * ((H + 255) / 256) < 4096 ? 1 : 0;
    p.offsets = (int*)(ws + off[0]); p.cursor = (int*)(ws + off[1]); p.ntiles = (int*)(ws + off[2]);
    p.tile_rec = (MoeTileRec*)(ws + off[3]);
    p.sorted_tok = (int*)(ws + off[6]); p.pos = (int*)(ws + off[7]);
    p.xq = (uint8_t*)(ws + off[8]); p.xs = (float*)(ws + off[9]);
    p.aq = (uint8_t*)(ws + off[10]); p.as = (float*)(ws + off[11]);
    p.o = (float*)(ws + off[12]);
    return moe_launch(p, first_stage, last_stage, (hipStream_t)stream) == 0 ? ATTN_OK : ATTN_ERR_LAUNCH;
}

extern "C" int moe_ffn_fp8(const void* x, const int* ids, const float* wts,
                           const void* w13, const float* s13, const void* w2, const float* s2,
                           void* y, int T, int H, int I, int E, int KTOP,
                           void* workspace, size_t workspace_bytes, void* stream) {
    return moe_ffn_fp8_ex(x, ids, wts, w13, s13, w2, s2, y, T, H, I, E, KTOP, workspace, workspace_bytes, 0, 4, 0, stream);
}

extern "C" int moe_ffn_fp8_static(const void* x, const int* ids, const float* wts,
                                  const void* w13, const float* s13, const void* w2, const float* s2,
                                  void* y, int T, int H, int I, int E, int KTOP, void* stream) {
    if (!x || !ids || !wts || !w13 || !s13 || !w2 || !s2 || !y) return ATTN_ERR_NULL_PTR;
    if (!sizes_ok(T, H, I, E, KTOP)) return ATTN_ERR_BAD_SHAPE;
    size_t off[13];
    if (moe_workspace_layout(T, H, I, E, KTOP, off) > kMoeStaticScratchBytes) return ATTN_ERR_TOO_LARGE;
    size_t have = 0;
    void* const scratch = moe_static_scratch(&have);      // cached per device after the first call; no allocation
    if (!scratch) return ATTN_ERR_LAUNCH;
    return moe_ffn_fp8_ex(x, ids, wts, w13, s13, w2, s2, y, T, H, I, E, KTOP, scratch, have, 0, 4, 0, stream);
}

extern "C" int moe_ffn_fp8_row_tiles(int rows, int row_tile) {
    if (rows < 0 || (row_tile != 0 && row_tile != 64 && row_tile != 128)) return -1;
    return moe_row_tiles(rows, row_tile ? row_tile : 128);
}

extern "C" double moe_ffn_fp8_flops_per_pair(int H, int I) {
    if (H <= 0 || I <= 0) return 0.0;
    return 6.0 * (double)H * (double)I;
}

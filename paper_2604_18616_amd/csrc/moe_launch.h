// Internal interface between the C-ABI translation unit (argument checks, workspace layout,
// no device code) and the MoE kernel translation unit.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

constexpr int kMoeBM = 64;   // smallest row tile (routed token slots of one expert) of the grouped products: sizes the tile tables

// What a workgroup of the grouped products needs to know about the expert its row tile belongs to, in one
// 16-byte load: the tile's own first row and row count follow from these by arithmetic (moe_row_tiles), so the
// chain of dependent loads in front of a workgroup's first copy is: number of tiles -> this record -> (gate/up
// only) the tokens of its rows.
struct MoeTileRec {
    int expert;               // the expert
    int row0;                 // its first sorted row
    int rows;                 // its number of rows
    int first;                // index of its first row tile
};

// Row tiles of an expert with cnt rows: tiles of bm rows and a remainder.  An expert with one full tile and
// at most 32 rows more gets a single tile of up to bm + 32 rows (one more 32-row MFMA block instead of a
// second copy of every weight tile: 13 % on the whole call where experts have about bm rows).  With two or
// more full tiles the remainder stays a tile of its own: measured, the short tiles then cost little (their
// weights are L2 hits) and fill the last round of workgroups, which equal long tiles leave mostly idle.
__host__ __device__ inline int moe_row_tiles(int cnt, int bm) {
    const int n = cnt / bm, r = cnt - n * bm;
    return (n == 1 && r <= 32) ? 1 : n + (r > 0 ? 1 : 0);
}

struct MoeParams {
    const __bf16* x; const int* ids; const float* wts;
    const uint8_t* w13; const float* s13; const uint8_t* w2; const float* s2;
    __bf16* y;
    int T, H, I, E, KTOP;
    int bm;                   // rows per tile for this call: 64 or 128
    int max_tiles;            // upper bound on the number of row tiles: ceil(T*KTOP / bm) + E
    int dn_narrow_ok;         // the grid of the down product is sized for 128-row column tiles (the kernel decides whether to use them)
    // workspace carve-up (all device pointers into the caller's workspace)
    int* offsets;             // [E + 1] first sorted row of each expert
    int* cursor;              // [E]     scatter cursors
    int* ntiles;              // [1]     row tiles in use
    MoeTileRec* tile_rec;     // [max_tiles] one record per row tile
    int* sorted_tok;          // [T*KTOP] token of each sorted row
    int* pos;                 // [T*KTOP] sorted row of slot (t, k), or -1 if the slot is not local
    uint8_t* xq; float* xs;   // [T, H] codes, [T, H/128] scales
    uint8_t* aq; float* as;   // [T*KTOP, I] codes, [T*KTOP, I/128] scales of the intermediate
    float* o;                 // [T*KTOP, H] down-projection rows
};

// Byte offsets of the workspace parts for given sizes; returns the total.
size_t moe_workspace_layout(int T, int H, int I, int E, int KTOP, size_t off[13]);

// Enqueue stages first..last of the path (0 route, 1 quantize x, 2 gate/up, 3 down, 4 combine) on
// `stream`.  Returns 0, or -1 if a launch was refused.
int moe_launch(const MoeParams& p, int first, int last, hipStream_t stream);

// Library-owned scratch memory of the allocation-free entry point: the address, on the CURRENT device, of a
// file-scope device array of *bytes bytes (looked up once per device, then cached); nullptr if the runtime
// cannot resolve it.  The array is shared by every call on that device.
constexpr size_t kMoeStaticScratchBytes = (size_t)128 << 20;
void* moe_static_scratch(size_t* bytes);

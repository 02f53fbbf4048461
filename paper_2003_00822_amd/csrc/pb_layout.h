// Internal: packed-weight layout and workspace carving shared by the host API
// and the kernels of this library (not part of the public ABI).
//
// Packed layout PB_LAYOUT_ROWMAJOR_V1: uint32 words, [bitlayer i][row r][word w],
// bitlayer 0 = sign layer (Section 3.2 / Algorithm 1 of the paper), bit (c % 32)
// of word c / 32 is the layer's bit for column c (Section 3.4: 32 values per
// word).  Rows are padded to `rows_p` and words per row to `cwp`; padding is 0.
#pragma once
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

#include "pb.h"

namespace pb {

constexpr int kWave = 64;
constexpr int kTileWords = 128;     // one matvec tile: 64 lanes x 2 words
constexpr int kRing = 8;            // weight tiles in flight per wave
constexpr int kMaxWavesPerWG = 8;
constexpr int kMetaInts = 16;       // per activation vector, in the workspace

struct Layout {
    int rows, cols, bits;
    int cw;        // words that hold real columns: ceil(cols / 32)
    int ws;        // words of one row handled by one wave (32, 64 or 128)
    int csplit;    // waves that share a row: cwp = ws * csplit
    int cwp;       // padded words per row
    int rpt;       // rows per tile = 128 / ws
    int rows_p;    // rows padded to a multiple of 4
    size_t layer_words;  // rows_p * cwp
};

inline bool make_layout(int rows, int cols, int bits, Layout *L)
{
    if (rows < 1 || cols < 1 || bits < 1 || bits > PB_MAX_BITS) return false;
    if (cols > PB_MAX_COLS) return false;
    L->rows = rows; L->cols = cols; L->bits = bits;
    L->cw = (cols + 31) / 32;
    int best_ws = 0, best_pad = 0;
    const int cand[3] = {128, 64, 32};
    const char *force = getenv("PB_TUNE_WS");
    for (int k = 0; k < 3; ++k) {
        int ws = cand[k];
        if (force && atoi(force) != ws) continue;
        int cs = (L->cw + ws - 1) / ws;
        if (cs > kMaxWavesPerWG) continue;
        int pad = cs * ws;
        if (best_ws == 0 || pad < best_pad) { best_ws = ws; best_pad = pad; }
    }
    if (best_ws == 0) return false;
    L->ws = best_ws;
    L->csplit = best_pad / best_ws;
    L->cwp = best_pad;
    L->rpt = kTileWords / best_ws;
    L->rows_p = (rows + 3) & ~3;
    L->layer_words = (size_t)L->rows_p * (size_t)L->cwp;
    return true;
}

inline size_t packed_bytes(const Layout &L) { return L.layer_words * (size_t)L.bits * sizeof(uint32_t); }

// Workspace: [meta: batch * kMetaInts int32][planes: batch * 32 * cwp uint32][gates: batch * rows fp32]
inline size_t ws_meta_off(const Layout &, int) { return 0; }
inline size_t ws_planes_off(const Layout &, int batch) { return ((size_t)batch * kMetaInts * 4 + 255) & ~(size_t)255; }
inline size_t ws_gates_off(const Layout &L, int batch)
{
    return (ws_planes_off(L, batch) + (size_t)batch * 32 * (size_t)L.cwp * 4 + 255) & ~(size_t)255;
}
inline size_t workspace_bytes(const Layout &L, int batch)
{
    return (ws_gates_off(L, batch) + (size_t)batch * (size_t)L.rows * 4 + 255) & ~(size_t)255;
}

}  // namespace pb

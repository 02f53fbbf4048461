// Internal: packed-weight layouts and workspace carving shared by the host API
// and the kernels of this library (not part of the public ABI).
//
// Both layouts store uint32 words of 32 columns each (Section 3.4 of the paper: 32
// values per word), bit (c % 32) of word c / 32 is the layer's bit for column c,
// bitlayer 0 = sign layer (Section 3.2 / Algorithm 1), one bitlayer after the other
// (`layer_words` apart) so that the first `bits_used` layers are one contiguous
// region.  Rows are padded to `rows_p` and words per row to `cwp`; padding is 0.
//
// PB_LAYOUT_ROWMAJOR_V1: [bitlayer][row][word].  Read by the AND + popcount kernel.
//
// PB_LAYOUT_TILE16_V1: [bitlayer][row tile of 16][chunk of 16 words][lane][4 words].
//   A 1 KB block holds 16 rows x 16 words in the order a wave of the matrix-core
//   kernel consumes it: lane l = 16 * kb + j (j = row in the tile, kb = 0..3) owns
//   the 16 bytes at l * 16, the words 16 * chunk + 4 * kb + t (t = 0..3) of row j.
//   One 16-byte load per lane fetches a whole block, fully coalesced, and word t of
//   every lane is the B operand of one 16x16x128 matrix instruction (row j, k-block kb).
//
// PB_LAYOUT_TILE16_GATES_V1: the same blocks for the fused gate matrix of an LSTM (rows = 4H
//   in gate order i, f, g, o): row tile t holds the four gate rows of the hidden units 4t .. 4t+3,
//   packed row 16 t + 4 (u % 4) + gate = matrix row gate * H + u.  All four pre-activations of
//   a hidden unit then end in one row tile, so the cell update can follow the product in
//   the same launch.
//
// PB_LAYOUT_TILE16_PAIRS_V1: the same blocks, but the words of the bitlayers (2p, 2p + 1) hold base-4 digits
//   d_c = 2 w_(2p)[c] + w_(2p+1)[c] instead of single bits: the word at the position of bitlayer 2p holds the digits of
//   the even columns of its 32 columns (d_c in bits c, c + 1), the word at the position of bitlayer 2p + 1 those of the
//   odd columns (d_c in bits c - 1, c).  Bitlayer 0 enters complemented (the digit 2 (1 - w_0) + w_1 of the sign
//   pair, Section 3.2's sign bitlayer with the scale of its neighbour).  `stored_bits` = bits rounded up to an even
//   number; a last single bitlayer is paired with zeros.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include "pb.h"

namespace pb {

constexpr int kWave = 64;
constexpr int kTileWords = 128;     // popcount kernel: one tile = 64 lanes x 2 words
constexpr int kRing = 8;            // popcount kernel: weight tiles in flight per wave
constexpr int kMaxWavesPerWG = 8;   // popcount kernel
constexpr int kMetaInts = 16;       // per activation vector, in the workspace

constexpr int kTileRows = 16;       // matrix-core kernel: rows per tile
constexpr int kChunkWords = 16;     // matrix-core kernel: words per row in one block
constexpr int kMaxSlices = 16;      // matrix-core kernel: waves (column slices) per workgroup
constexpr int kMaxColsTile16 = 32768;     // 16 slices of 2048 columns
// merged bitlayer pairs (digit products up to 9): a quarter sum stays below 4369 * 9 * 32768 < 2^31, so pairs cover
// every width the tiled layouts have
constexpr int kMaxColsPairs = 32768;
// Bitlayer pairs whose sums the matrix-core kernel accumulates in one set of registers (pair p of a group counts
// 4^(last - p)): with five, a register stays below 9 * 2048 * 341 < 2^24 and the half sums of a row below
// 17 * 9 * 32768 * 341 < 2^31.
constexpr int kPairGroup = 5;

// Batches on rows wider than the digit rows that the waves of a workgroup of the matrix-core kernel hold are
// covered in several passes over the columns: at most `cap` chunks of 512 columns per pass (what eight waves hold:
// kSplitChunks4 with four operands per wave, kSplitChunks8 with eight), the chunks shared out evenly.  The launcher
// sizes the workgroup with these and the kernel finds its slice with them.
constexpr int kSplitChunks4 = 16, kSplitChunks8 = 8;
__host__ __device__ inline int split_parts(int cq, int cap) { return (cq + cap - 1) / cap; }
__host__ __device__ inline int split_chunks_per_part(int cq, int cap)
{
    const int parts = split_parts(cq, cap);
    return (cq + parts - 1) / parts;
}

struct Layout {
    uint32_t layout;
    int rows, cols, bits;
    int stored_bits;   // bitlayers that the packed buffer has room for (bits, or the next even number: pairs layout)
    int cw;        // words that hold real columns: ceil(cols / 32)
    int cwp;       // padded words per row
    int rows_p;    // padded rows
    size_t layer_words;  // rows_p * cwp
    // PB_LAYOUT_ROWMAJOR_V1
    int ws;        // words of one row handled by one wave (32, 64 or 128)
    int csplit;    // waves that share a row: cwp = ws * csplit
    int rpt;       // rows per tile = 128 / ws
    // PB_LAYOUT_TILE16_V1
    int rt_count;  // row tiles: rows_p / 16
    int cq;        // chunks per row: cwp / 16
    int gate_h;    // PB_LAYOUT_TILE16_GATES_V1: H = rows / 4 (rows are stored gate-interleaved), else 0
};

__host__ __device__ inline bool is_pairs(uint32_t layout) { return layout == PB_LAYOUT_TILE16_PAIRS_V1; }
inline bool is_tile16(uint32_t layout)
{
    return layout == PB_LAYOUT_TILE16_V1 || layout == PB_LAYOUT_TILE16_GATES_V1 || is_pairs(layout);
}

// PB_LAYOUT_TILE16_GATES_V1: packed row of matrix row r, and back (-1 = a padding row).
__host__ __device__ inline int gates_packed_row(int r, int H)
{
    const int gate = r / H, u = r - gate * H;
    return (u >> 2) * 16 + (u & 3) * 4 + gate;
}
__host__ __device__ inline int gates_matrix_row(int pr, int H)
{
    const int u = (pr >> 4) * 4 + ((pr >> 2) & 3), gate = pr & 3;
    return u < H ? gate * H + u : -1;
}

inline bool make_layout(uint32_t layout, int rows, int cols, int bits, Layout *L)
{
    if (rows < 1 || cols < 1 || bits < 1 || bits > PB_MAX_BITS) return false;
    if (cols > PB_MAX_COLS) return false;
    L->layout = layout;
    L->rows = rows; L->cols = cols; L->bits = bits;
    L->stored_bits = is_pairs(layout) ? (bits + 1) & ~1 : bits;
    L->cw = (cols + 31) / 32;
    L->ws = L->csplit = L->rpt = L->rt_count = L->cq = L->gate_h = 0;
    if (layout == PB_LAYOUT_ROWMAJOR_V1) {
        int best_ws = 0, best_pad = 0;
        const int cand[3] = {128, 64, 32};
        for (int k = 0; k < 3; ++k) {
            int ws = cand[k];
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
    } else if (is_tile16(layout)) {
        if (cols > kMaxColsTile16) return false;
        L->cq = (L->cw + kChunkWords - 1) / kChunkWords;
        L->cwp = L->cq * kChunkWords;
        if (layout == PB_LAYOUT_TILE16_GATES_V1) {
            if (rows % 4 != 0) return false;
            L->gate_h = rows / 4;
            L->rt_count = (L->gate_h + 3) / 4;       // four hidden units (16 gate rows) per tile
        } else {
            L->rt_count = (rows + kTileRows - 1) / kTileRows;
        }
        L->rows_p = L->rt_count * kTileRows;
    } else {
        return false;
    }
    L->layer_words = (size_t)L->rows_p * (size_t)L->cwp;
    return true;
}

// Strides (in words) of the tiled layout: between the bitlayers of one row tile and between row tiles.
// (Bitlayer-major; keeping the bitlayers of a row tile next to each other instead measured the same speed.)
inline size_t tile16_layer_stride(const Layout &L) { return L.layer_words; }
inline size_t tile16_rowtile_stride(const Layout &L) { return (size_t)L.cq * 256; }

// Position (in words) of word w of PACKED row r of bitlayer `layer`.
__host__ __device__ inline size_t word_index(uint32_t layout, int cwp, size_t layer_words, int layer, int r, int w)
{
    if (layout == PB_LAYOUT_ROWMAJOR_V1) return (size_t)layer * layer_words + (size_t)r * (size_t)cwp + (size_t)w;
    const size_t cq = (size_t)(cwp / kChunkWords);
    const int lane = ((w % kChunkWords) / 4) * kTileRows + (r % kTileRows);
    const size_t in_block = (size_t)lane * 4 + (size_t)(w % 4);
    const size_t rt = (size_t)(r / kTileRows), q = (size_t)(w / kChunkWords);
    return (size_t)layer * layer_words + (rt * cq + q) * 256 + in_block;
}

inline size_t packed_bytes(const Layout &L) { return L.layer_words * (size_t)L.stored_bits * sizeof(uint32_t); }

// PB_LAYOUT_TILE16_PAIRS_V1: the two words (even columns, odd columns) of the digits 2 hi + lo of 32 columns, and back.
__host__ __device__ inline void digits_of_pair(uint32_t hi, uint32_t lo, uint32_t *even, uint32_t *odd)
{
    *even = (lo & 0x55555555u) | ((hi << 1) & 0xAAAAAAAAu);
    *odd = ((lo >> 1) & 0x55555555u) | (hi & 0xAAAAAAAAu);
}
__host__ __device__ inline void pair_of_digits(uint32_t even, uint32_t odd, uint32_t *hi, uint32_t *lo)
{
    *hi = ((even >> 1) & 0x55555555u) | (odd & 0xAAAAAAAAu);
    *lo = (even & 0x55555555u) | ((odd << 1) & 0xAAAAAAAAu);
}

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

// Host-side probe of the packed-layout arithmetic in csrc/pb_layout.h (compiled by tests/test_layout_host.py with
// g++; the header's functions are plain C++ once the HIP qualifiers are defined away).
#include <stdint.h>
#include "pb_layout.h"

extern "C" {

// fills out[0..9] = {cw, cwp, rows_p, rt_count, cq, gate_h, ws, csplit, rpt, ok}, returns layer_words
long long probe_layout(unsigned layout, int rows, int cols, int bits, int *out)
{
    pb::Layout L;
    const bool ok = pb::make_layout(layout, rows, cols, bits, &L);
    out[9] = ok ? 1 : 0;
    if (!ok) return -1;
    out[0] = L.cw; out[1] = L.cwp; out[2] = L.rows_p; out[3] = L.rt_count; out[4] = L.cq; out[5] = L.gate_h;
    out[6] = L.ws; out[7] = L.csplit; out[8] = L.rpt;
    return (long long)L.layer_words;
}

long long probe_word_index(unsigned layout, int cwp, long long layer_words, int layer, int r, int w)
{
    return (long long)pb::word_index(layout, cwp, (size_t)layer_words, layer, r, w);
}

int probe_gates_packed_row(int r, int H) { return pb::gates_packed_row(r, H); }
int probe_gates_matrix_row(int pr, int H) { return pb::gates_matrix_row(pr, H); }
long long probe_packed_bytes(unsigned layout, int rows, int cols, int bits)
{
    pb::Layout L;
    if (!pb::make_layout(layout, rows, cols, bits, &L)) return -1;
    return (long long)pb::packed_bytes(L);
}
long long probe_workspace_bytes(unsigned layout, int rows, int cols, int bits, int batch)
{
    pb::Layout L;
    if (!pb::make_layout(layout, rows, cols, bits, &L)) return -1;
    return (long long)pb::workspace_bytes(L, batch);
}

// limits that the accumulator bounds depend on: {columns of a tiled matrix, columns with merged bitlayer pairs, column slices per row, bitlayer pairs that share accumulators}
void probe_limits(int *out)
{
    out[0] = pb::kMaxColsTile16;
    out[1] = pb::kMaxColsPairs;
    out[2] = pb::kMaxSlices;
    out[3] = pb::kPairGroup;
}

// PB_LAYOUT_TILE16_PAIRS_V1: the digit words of a bitlayer pair and back; out = {even, odd, upper, lower}
void probe_pair_digits(unsigned upper, unsigned lower, unsigned *out)
{
    pb::digits_of_pair(upper, lower, &out[0], &out[1]);
    pb::pair_of_digits(out[0], out[1], &out[2], &out[3]);
}

// wide rows in several passes of at most cap chunks: out = {passes, chunks per pass} for a row of cq chunks
void probe_split(int cq, int cap, int *out)
{
    out[0] = pb::split_parts(cq, cap);
    out[1] = pb::split_chunks_per_part(cq, cap);
}
void probe_split_caps(int *out)
{
    out[0] = pb::kSplitChunks4;
    out[1] = pb::kSplitChunks8;
}

}  // extern "C"

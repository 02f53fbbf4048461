/*
 * pb.h -- C ABI of the MI355X (gfx950) PrecisionBatching hot path.
 *
 * The library computes the bit-decomposed quantized matrix product of
 * "Quantized Neural Network Inference with Precision Batching"
 * (arXiv 2003.00822): a B-bit weight matrix is stored as B packed 1-bit
 * bitlayers (Section 3.2, Algorithm 1), fp32 activations are converted to
 * 32-bit fixed point and split into bit planes that are batched as extra
 * columns (Section 3.1, Algorithm 2), products are AND + population count on
 * packed words (Section 3.4), and the per-bitlayer results are scaled and
 * accumulated over the first `bits_used` bitlayers, a number chosen per call
 * (abstract; Section 1).
 *
 * Conventions
 *  - Every pointer is a DEVICE pointer unless its comment says "host".
 *  - Matrices are dense row-major.  Device pointers must be 16-byte aligned.
 *  - The caller owns every buffer, including `packed` and `workspace`; the
 *    library allocates and frees nothing, keeps no state and never
 *    synchronises.  All work is enqueued on `stream` (a hipStream_t passed as
 *    void*, NULL = the default stream); calls on different streams may run
 *    concurrently as long as they use different workspaces and outputs.
 *  - Every function returns PB_OK (0) or a negative pb_status; nothing
 *    throws or aborts.  Argument errors are detected on the host before
 *    anything is launched.  A HIP launch failure returns PB_EHIP
 *    (pb_last_hip_error() gives the HIP code); a fault inside a kernel
 *    surfaces at the caller's next synchronisation, as for any HIP work.
 *  - Weights and activations are assumed finite; a NaN activation converts
 *    to 0 and +-inf saturates (see pb_matmul).
 */
#ifndef PB_H
#define PB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum pb_status {
    PB_OK = 0,
    PB_EINVAL = -1, /* null pointer, non-positive size, bits / bits_used / batch out of range */
    PB_EALIGN = -2, /* a device pointer is not 16-byte aligned */
    PB_ESIZE = -3,  /* shape beyond what the kernels support (see PB_MAX_*) */
    PB_EHIP = -4    /* a HIP call failed */
} pb_status;

#define PB_MAX_BITS 16       /* stored bitlayers B, 1..16 (Section 1: "1-16 bit execution") */
#define PB_MAX_COLS 32768    /* columns of one weight matrix */
#define PB_MAX_BATCH 4096    /* activation vectors per call */

/* Packed layouts (opaque to the caller; pb_unpack reads either).
 * PB_LAYOUT_TILE16_V1   16-row x 512-column blocks in the order the matrix-core kernel streams them; the
 *                       default.  The product runs as FP4 matrix
 *                       instructions on the bitlayers and planes (two of each per operand element, as
 *                       base-4 digits), exact in fp32 accumulators.
 * PB_LAYOUT_ROWMAJOR_V1 [bitlayer][row][word]; read by the AND + popcount kernel (Section 3.4 taken
 *                       literally), kept as the measured alternative. */
#define PB_LAYOUT_ROWMAJOR_V1 0x50420001u
#define PB_LAYOUT_TILE16_V1 0x50420002u
/* PB_LAYOUT_TILE16_GATES_V1  the tiled layout for the fused gate matrix of an LSTM (rows = 4H, gate order
 *                       i, f, g, o): the four gate rows of a hidden unit share a row tile, so that
 *                       pb_lstm_cell runs as ONE launch.  Every other call works on it too and sees the
 *                       rows in their matrix order.  Chosen by the caller (pb_desc_init_layout). */
#define PB_LAYOUT_TILE16_GATES_V1 0x50420003u
/* PB_LAYOUT_TILE16_PAIRS_V1  the tiled layout for callers that serve batches: the bitlayers (2p, 2p + 1) are
 *                       stored together as base-4 digits 2 w_(2p) + w_(2p+1), two bits per column (the digits
 *                       of the even columns of a word in the block of bitlayer 2p, those of the odd columns in
 *                       the block of bitlayer 2p + 1; bitlayer 0 enters complemented; an odd number of
 *                       bitlayers is stored as the next even number, the last one paired with zeros, and
 *                       pb_packed_bytes says so).  The matrix-core kernel then builds a weight operand of two
 *                       bitlayers with six instead of ten operations: about 10 % faster from batch 16 on.
 *                       Every call works on it (not pb_lstm_cell's single launch); with one vector it is slower than
 *                       PB_LAYOUT_TILE16_V1, because an odd bits_used reads one bitlayer more.  Chosen by the
 *                       caller (pb_desc_init_layout). */
#define PB_LAYOUT_TILE16_PAIRS_V1 0x50420004u

/* Shape and format of one packed weight matrix (host struct, plain data).
 * bits      B, the number of stored bitlayers = two's-complement width of the
 *           weight codes, sign layer included (the paper's "PBatch-n" stores
 *           n+1 layers: bits = n+1; Table 1 caption).
 * frac_bits f, position of the activations' fixed point (Section 3.1: 16, "may
 *           be changed").
 * act_bits  k, number of activation bit planes (Algorithm 2: 32).
 * layout    tag of the packed layout (PB_LAYOUT_*), filled by pb_desc_init. */
typedef struct pb_desc {
    int32_t rows, cols, bits;
    int32_t frac_bits;
    int32_t act_bits;
    uint32_t layout;
} pb_desc;

/* Fill *d (host) for a rows x cols matrix with `bits` bitlayers and the
 * defaults f = 16, k = 32.  pb_desc_init picks PB_LAYOUT_TILE16_V1 (the layout
 * of the matrix-core kernel, the fastest for every shape the interface
 * allows); pb_desc_init_layout takes the layout from the caller.
 * PB_EINVAL / PB_ESIZE on bad shapes or a layout that does not fit the shape. */
int pb_desc_init(pb_desc *d, int rows, int cols, int bits);
int pb_desc_init_layout(pb_desc *d, int rows, int cols, int bits, uint32_t layout);

/* Bytes the caller must allocate for `packed` (all B bitlayers, padded),
 * and for `workspace` of a call with `batch` activation vectors (bit planes,
 * plane statistics, and for pb_lstm_cell the gate pre-activations).
 * Return 0 if the descriptor is invalid. */
size_t pb_packed_bytes(const pb_desc *d);
size_t pb_workspace_bytes(const pb_desc *d, int batch);

/* Algorithm 1 (preprocessing, offline): quantize W to B-bit codes on a
 * symmetric linear grid, q = round_half_even(W / step), step = max|W| /
 * (2^(B-1) - 1) (Section 3.3; step = max|W| for B = 1, step = 1 for W = 0),
 * split the two's-complement codes into B bitlayers, sign layer first
 * (Section 3.2), pack 32 columns per word (Section 3.4) and write the layer
 * scales scales[i] = step * s_i, s_0 = -2^(B-1), s_i = 2^(B-1-i).
 *   W       [rows][cols] fp32, read only
 *   packed  pb_packed_bytes() bytes, written (opaque layout, see pb_unpack)
 *   scales  [bits] fp32, written
 * Launches a few kernels on `stream`; nothing is returned to the host. */
int pb_quantize_pack(const float *W, int rows, int cols, int bits, void *packed, float *scales, void *stream);

/* The same for a descriptor the caller filled (pb_desc_init_layout): packs into
 * d->layout.  pb_quantize_pack(W, rows, cols, bits, ...) is this call on the
 * descriptor pb_desc_init(rows, cols, bits) gives. */
int pb_quantize_pack_desc(const float *W, const pb_desc *d, void *packed, float *scales, void *stream);

/* The other quantizers of Section 3.3, same outputs as pb_quantize_pack_desc (q = B-bit codes on a linearly spaced
 * grid, scales[i] = step * s_i):
 *   PB_QUANT_SYMMETRIC    step = max|W| / (2^(B-1) - 1): what pb_quantize_pack does
 *   PB_QUANT_RANGE        the printed formula, step = (max W - min W) / 2^(B-1), codes clamped to the B-bit range
 *   PB_QUANT_SIGN         "for quantizing to 1 bit ... exclude representing 0": q = +1 (W >= 0) or -1,
 *                         step = mean |W|; needs bits = 2 (sign layer + one magnitude layer)
 *   PB_QUANT_CLIP_SEARCH  "optimize over a clipping threshold": the symmetric quantizer with the threshold
 *                         max|W| * k / 32 (k = 1..32) whose mean |W - step * q| is smallest
 * PB_EINVAL for an unknown quantizer or PB_QUANT_SIGN with bits != 2. */
typedef enum pb_quantizer {
    PB_QUANT_SYMMETRIC = 0,
    PB_QUANT_RANGE = 1,
    PB_QUANT_SIGN = 2,
    PB_QUANT_CLIP_SEARCH = 3
} pb_quantizer;
int pb_quantize_pack_mode(const float *W, const pb_desc *d, int quantizer, void *packed, float *scales, void *stream);

/* Inverse of the packing, for checking: q[r][c] = the B-bit code stored for
 * element (r, c), sign-extended to int32.  q: [rows][cols], written. */
int pb_unpack(const void *packed, const pb_desc *d, int32_t *q, void *stream);

/* Algorithm 2 (inference).  For each of the `batch` activation vectors:
 *   x_q = trunc(x * 2^f) as a k-bit two's-complement integer (saturating;
 *   NaN -> 0), split into k bit planes with weights 2^j and -2^(k-1);
 *   A_i[r] = sum_j c_j * popcount(row r of bitlayer i AND plane j)  (exact, int64; computed as
 *            AND + popcount or as an exact matrix product of the same bits, depending on the layout)
 *   Y[r]   = fp32( sum_{i < bits_used} scales[i] * A_i[r] * 2^-f )  (sum in fp64; where two adjacent
 *            scales are in the ratio of Algorithm 1 the tiled layouts may add the pair's integers first,
 *            see pb_matmul_acc_pairs: the same sum up to the fp64 rounding of its terms)
 * Only the first `bits_used` bitlayers (sign layer and the next bits_used-1)
 * are read: the accuracy / speed knob of the abstract.
 *   packed, scales  as written by pb_quantize_pack (scales may be any fp32 values)
 *   d               host descriptor
 *   X               [batch][cols] fp32, read only
 *   Y               [batch][rows] fp32, written
 *   workspace       pb_workspace_bytes(d, batch) bytes, overwritten
 * The activation conversion and bit transposition are part of the call. */
int pb_matmul(const void *packed, const float *scales, const pb_desc *d, int bits_used, const float *X, int batch,
              float *Y, void *workspace, void *stream);

/* pb_matmul for callers that cannot allocate device memory (code under HIP
 * graph capture, serving loops that own no buffers, harnesses that forbid
 * hipMalloc): the same kernels and the same result as pb_matmul, with the
 * workspace (bit planes and plane statistics of the activations, which only the
 * PB_LAYOUT_ROWMAJOR_V1 kernels use) in a device array of
 * PB_STATIC_SCRATCH_BYTES that the library holds on every GPU it runs on until
 * the process ends.  Allocates, frees and synchronises nothing.
 * PB_ESIZE if pb_workspace_bytes(d, batch) exceeds PB_STATIC_SCRATCH_BYTES
 * (a 4096 x 4096 matrix: up to 63 vectors; 32768 columns: up to 14).
 * All calls on one GPU share that array: calls that may overlap in time on one
 * GPU (different streams, different threads) race on it and must be serialised by
 * the caller; use pb_matmul with separate workspaces for concurrent calls. */
#define PB_STATIC_SCRATCH_BYTES (2u << 20)
int pb_matmul_static(const void *packed, const float *scales, const pb_desc *d, int bits_used, const float *X, int batch,
                     float *Y, void *stream);

/* pb_matmul with the layer's bias and nonlinearity applied before the store (the paper replaces each linear
 * layer and keeps the nonlinearities in fp32, Sections 4.2-4.3):
 *   Y[n][r] = act( fp32(sum_i scales[i] * A_i[r] * 2^-f) + bias[r] ),  act = identity or max(., 0).
 *   bias  [rows] fp32 or NULL (read only);  act  a pb_activation. */
typedef enum pb_activation { PB_ACT_NONE = 0, PB_ACT_RELU = 1 } pb_activation;
int pb_matmul_bias_act(const void *packed, const float *scales, const pb_desc *d, int bits_used, const float *X,
                       int batch, const float *bias, int act, float *Y, void *workspace, void *stream);

/* Same product, but returns the exact integer accumulators instead of Y:
 * A[i][n][r] = sum_c bit_i[r][c] * x_q[n][c], int64, for i < bits_used.
 * A: [bits_used][batch][rows], written. */
int pb_matmul_acc(const void *packed, const pb_desc *d, int bits_used, const float *X, int batch, int64_t *A,
                  void *workspace, void *stream);

/* The accumulators as the matrix-core kernel holds them when it multiplies two
 * adjacent bitlayers in one instruction (Section 3.4: bitlayers stacked in one
 * operation; the scales of Algorithm 1 halve from bitlayer to bitlayer and the
 * sign bitlayer has scale -2 s_1, so s_(i) A_(i) + s_(i+1) A_(i+1) =
 * s_(i+1) (+-2 A_(i) + A_(i+1))).  The units are the pairs (0, 1), (2, 3), ...
 * and a last single bitlayer if bits_used is odd: P[0] = -2 A_0 + A_1 (A_0 if
 * bits_used is 1), P[p] = 2 A_(2p) + A_(2p+1), P[last] = A_(bits_used-1) for a
 * single one.
 * A: [(bits_used + 1) / 2][batch][rows] int64, written.  Tiled layouts only
 * (PB_EINVAL for PB_LAYOUT_ROWMAJOR_V1).  pb_matmul with more than one vector
 * takes this route by itself when scales[0] == -2 * scales[1] and scales[2p] ==
 * 2 * scales[2p + 1] hold for every pair, else it multiplies bitlayer by
 * bitlayer. */
int pb_matmul_acc_pairs(const void *packed, const pb_desc *d, int bits_used, const float *X, int batch, int64_t *A,
                        void *workspace, void *stream);

/* The two halves of pb_matmul, for callers that apply several weight matrices
 * to the same activations (or that time the halves separately):
 * pb_act_prep converts X to fixed point and writes its bit planes and plane
 * statistics into `workspace` (Algorithm 2, x_q = Int(x * 2^f), and the bitwise
 * transpose of Section 3.4); pb_matmul_prepared runs the product (AND +
 * popcount on PB_LAYOUT_ROWMAJOR_V1, the matrix-core kernel on the tiled
 * layouts, which then builds its operands from the planes) and the
 * scale-accumulation on planes left there by pb_act_prep.
 * The planes are laid out for the descriptor they were made with: the
 * descriptor of pb_matmul_prepared must have the same cols, LAYOUT, frac_bits
 * and act_bits, and the call the same batch (the distance between two planes
 * is the padded row length of the layout; another layout would read other
 * words, and nothing can check this).  Matrices that differ in rows and bits
 * only may share one pb_act_prep.
 * pb_matmul(...) computes the same Y as pb_act_prep(...) followed by
 * pb_matmul_prepared(...). */
int pb_act_prep(const pb_desc *d, const float *X, int batch, void *workspace, void *stream);
int pb_matmul_prepared(const void *packed, const float *scales, const pb_desc *d, int bits_used, int batch, float *Y,
                       void *workspace, void *stream);

/* The fixed-point activations alone (Algorithm 2, x_q = Int(x * 2^f)), for
 * checking: xq [batch][cols] int32, written; workspace as for pb_matmul
 * (the bit planes are left in it). */
int pb_fixed_point(const pb_desc *d, const float *X, int batch, int32_t *xq, void *workspace, void *stream);

/* One LSTM cell step on top of pb_matmul (Sections 4.2-4.3: the LSTM's input
 * and hidden linear maps run through the quantized product, nonlinearities in
 * fp32).  The packed matrix is the fused gate matrix, rows = 4H in gate order
 * (input, forget, cell, output), cols = I + H, applied to [x_t ; h_prev]:
 *   g = W [x_t ; h_prev] + bias,  c' = sigmoid(g_f) c + sigmoid(g_i) tanh(g_g),
 *   h' = sigmoid(g_o) tanh(c').
 *   x_t [batch][I], h_prev, c_prev [batch][H], bias [4H] or NULL: read only
 *   h_out, c_out [batch][H]: written (may alias h_prev / c_prev)
 *   input_size = I; H = d->rows / 4; d->cols must equal I + H.
 * With PB_LAYOUT_TILE16_GATES_V1 the product and the cell update are one launch, unless h_out overlaps
 * h_prev (every workgroup reads all of h_prev, so an in-place update has to wait for the whole product:
 * it then runs as two launches, like the other layouts). */
int pb_lstm_cell(const void *packed, const float *scales, const pb_desc *d, int bits_used, const float *x_t,
                 int input_size, const float *h_prev, const float *c_prev, const float *bias, float *h_out,
                 float *c_out, int batch, void *workspace, void *stream);

/* Text for a pb_status; the HIP error code of the last PB_EHIP on this thread. */
const char *pb_strerror(int status);
int pb_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PB_H */

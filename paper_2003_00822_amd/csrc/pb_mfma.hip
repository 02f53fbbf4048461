// The hot kernel on the matrix cores: the whole inference path of Algorithm 2 of the
// paper in one launch -- x_q = Int(x * 2^f), the bitwise transpose into bit planes
// (Section 3.4), the 1-bit products of Section 3.1 with the planes of a vector
// batched as the second matrix operand ("one batched matrix product"), the plane
// weights [-2^31, 2^30 .. 2^0] and the scale-accumulation over the first `bits_used`
// bitlayers (the run-time knob of the abstract).
//
// Why the matrix cores: AND + popcount costs two vector-ALU lane operations per
// (32-bit weight word, plane); with 32 planes that is four times what the ALUs of
// this chip can do while HBM delivers the words.  The same inner products are a
// dense contraction, and V_MFMA_SCALE_F32_16X16X128_F8F6F4 on FP4 (E2M1) operands
// does 32768 multiply-adds per instruction with exact results.
//
// Two planes per operand row.  E2M1 holds 0, 0.5, 1.0 and 1.5 as the codes 0, 1, 2, 3,
// so the two adjacent planes 2 i and 2 i + 1 of the activations travel as ONE row of
// base-4 digits d = b_(2i) + 2 b_(2i+1) (FP4 code = d, value d / 2): the 32 planes of a
// vector are the 16 rows of one A operand and the plane weights become 4^i.  The weight
// bit is the code 2.0, so every product is the digit itself (0 .. 3), the fp32
// accumulators hold integers below 2^24 and every sum is exact.
// The sign plane: digit 15 (bits 31, 30) is the signed one, -2 b_31 + b_30, and E2M1 has
// the values 0, 0.5, -1.0, -0.5 too (codes 0000, 0001, 1010, 1001): the two's-complement
// value is sum_i 4^i digit_i with that one digit signed, nothing to correct afterwards.
//
// Two bitlayers per instruction.  The scales of Algorithm 1 halve from one bitlayer to the next, so
// s_(i) A_(i) + s_(i+1) A_(i+1) = s_(i+1) (2 A_(i) + A_(i+1)): the weight operand carries the base-4 digit
// 2 w_(i) + w_(i+1) (FP4 code = digit again) and one instruction does the work of two: the pairs are (0, 1),
// (2, 3), ... and a last single bitlayer if bits_used is odd.  The sign bitlayer has the scale -2 s_1, so its
// pair needs the digit w_1 - 2 w_0 = (2 (1 - w_0) + w_1) - 2: the bits of bitlayer 0 are complemented and
// 2 * sum_c x_q[c] is subtracted, a sum that one more chain of instructions against an operand of digits 1
// delivers once per call.  Pair p then counts 4 times pair p + 1: the block scale of the weight operand (a power
// of two per instruction) supplies that factor, and up to five pairs of a row tile add up in the same registers.
// The kernel checks scales[0] == -2 scales[1], scales[i] == 2 scales[i + 1] itself and multiplies bitlayer by
// bitlayer when that does not hold (any other scales are legal input).
// PB_LAYOUT_TILE16_PAIRS_V1 stores those digits instead of the bits (template flag IL below).
//
// Operands.  A (16 x 128) = 16 digit rows x 128 columns, B (128 x 16) = 128 columns x
// 16 weight rows, D (16 x 16): lane l of D holds row j = l % 16 of the weights and
// the operand rows 4 * (l / 16) + c in its four registers c (rows 0-7 carry the even
// digits, rows 8-15 the odd ones, see digit_of_row), so the digit weighting is
// arithmetic inside a lane.  A lane's B operand is 32 columns of one weight row = ONE
// packed word; register r, nibble n of both operands is column 4 n + r of the word:
//     b0 = (w << 2) & 0x44444444   b1 = (w << 1) & 0x44444444
//     b2 = w & 0x44444444          b3 = (w >> 1) & 0x44444444
//
// Mapping.  A wave owns a slice of the columns (NQ chunks of 512) for its whole life
// and keeps the digit rows of that slice in registers; it streams the 1 KB
// blocks of its slice (see pb_layout.h) for row tile after row tile and bitlayer
// after bitlayer with 16-byte loads, several blocks in flight.  The waves of a
// workgroup are the slices of one row; their per-(row, bitlayer) sums meet in LDS
// through integer atomics, once per row tile, and one wave applies the layer scales
// and stores.  All integer results are exact, so they do not depend on the schedule.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include <type_traits>

#include "pb_kernels.h"

namespace pb {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// The arguments that the first memory requests of a wave depend on are the kernel's leading scalar parameters: those
// (fourteen dwords) the hardware loads into registers before a wave starts (kernel-argument preload), so the requests
// need not wait for a round trip to the argument buffer.  The rest travels as one structure.
struct MfmaHead {
    const uint32_t *packed;
    const float *X0;            // activations: row n is [X0[n][0..cols0) ; X1[n][0..cols1)]
    uint32_t packed_bytes;      // (below 2^32: the blocks are addressed with 32-bit offsets)
    uint32_t flags;             // kPlanesGiven: bit planes already in memory (prepared mode); kSecondPart: X1 is given
    int cols0;
    int batch;
    uint32_t layer_step, round_step;   // bytes from one bitlayer of a row tile to the next, from one row tile to the next
    int rounds_per_wg;          // row tiles per workgroup
    int rt_count, cq;
    int m;                      // bitlayers to accumulate
};
constexpr uint32_t kPlanesGiven = 1, kSecondPart = 2;
struct MfmaArgs {
    const float *X1;
    const uint32_t *planes;     // non-null: bit planes already in memory [batch][32][cwp] (prepared mode)
    const float *scales;
    float *Y;
    long long *A;
    int pairs_out;              // A receives the sums of the bitlayer pairs (-2 A_0 + A_1, 2 A_(2p) + A_(2p+1)) instead of every A_i
    const float *bias;          // [rows] or null: added to the fp32 result
    const float *c_prev;        // non-null: LSTM cell update instead of the store of Y (gate-interleaved rows)
    float *h_out, *c_out;
    int relu;                   // max(., 0) before the store of Y
    int gate_h;                 // gate-interleaved rows: H (packed row 16 t + 4 (u % 4) + gate = row gate * H + u), else 0
    int cols1;
    int R, cwp;
    float fscale;               // 2^frac_bits
    int imin, imax;             // range of the act_bits-bit fixed-point values
    double out_scale;           // 2^-frac_bits
};

// x_q = Int(x * 2^f) as a k-bit two's-complement value: toward zero, saturating, NaN -> 0.  V_CVT_I32_F32 does
// exactly that for k = 32 (out-of-range inputs saturate, NaN converts to 0); narrower k clamp the integer.
template <bool NARROW>
__device__ __forceinline__ int32_t to_fixed_point(float x, float fscale, int32_t imin, int32_t imax)
{
    int32_t r;
    const float p = x * fscale;   // exact: a power of two
    asm("v_cvt_i32_f32 %0, %1" : "=v"(r) : "v"(p));
    if constexpr (NARROW)
        asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(r), "v"(imin), "v"(imax));   // imin <= imax: the clamp
    return r;
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_mov(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, CTRL, 0xf, 0xf, true);
}

// value of lane (l ^ J) for J < 16, inside each row of 16 lanes, on the vector ALU alone (DPP modifiers)
template <int J>
__device__ __forceinline__ uint32_t row_xor(uint32_t v)
{
    if constexpr (J == 8) return dpp_mov<0x128>(v);                     // row_ror:8
    else if constexpr (J == 4) return dpp_mov<0x1B>(dpp_mov<0x141>(v)); // row_half_mirror (l ^ 7), then quad_perm [3,2,1,0] (l ^ 3)
    else if constexpr (J == 2) return dpp_mov<0x4E>(v);                 // quad_perm [2,3,0,1]
    else return dpp_mov<0xB1>(v);                                       // quad_perm [1,0,3,2]
}

// z + (z of the lane D lanes away, D = 16 or 32), in both lanes
template <int D>
__device__ __forceinline__ double add_across(double z)
{
    const unsigned long long b = (unsigned long long)__double_as_longlong(z);
    const uint32_t lo = (uint32_t)b, hi = (uint32_t)(b >> 32);
    // the swap leaves (own, partner's) in one half of the lanes and (partner's, own) in the other
    const auto l = D == 16 ? __builtin_amdgcn_permlane16_swap(lo, lo, false, false)
                           : __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
    const auto h = D == 16 ? __builtin_amdgcn_permlane16_swap(hi, hi, false, false)
                           : __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
    return __longlong_as_double((long long)(((unsigned long long)h[0] << 32) | l[0])) +
           __longlong_as_double((long long)(((unsigned long long)h[1] << 32) | l[1]));
}

// Row order of the A operand.  The sixteen base-4 digits of a value travel as FP4 codes in two words: E = the even
// digits (x & 0x33333333: nibble k = digit 2 k) and O = the odd ones ((x >> 2) & 0x33333333: nibble k = digit
// 2 k + 1).  Operand row i is nibble i of the pair (E, O): rows 0-7 hold the digits 0, 2, .., 14 and rows 8-15 the
// digits 1, 3, .., 15.
__device__ __forceinline__ int digit_of_row(int i) { return ((i & 7) << 1) | (i >> 3); }

// x_q (k-bit two's complement, sign-extended) -> the FP4 codes of its sixteen digits, nibble i = digit
// digit_of_row(i); code = digit (value digit / 2), except for digit 15, the signed one (-2 b31 + b30: values
// 0, 1, -2, -1 = codes 0000, 0001, 1010, 1001), which a byte table indexed by the two top bits supplies.
// PK = 2, 4: x holds PK values of 32 / PK bits (activations of at most 16 / 8 bits, Section 3.1), each with its
// own signed top digit: the nibbles of (E, O) are then the digits of PK vectors, 8 / PK even and 8 / PK odd ones each.
template <int PK>
__device__ __forceinline__ uint2 digit_codes(uint32_t x)
{
    const uint32_t e = x & 0x33333333u;
    const uint32_t o = (x >> 2) & 0x33333333u;
    // the top two bits of every value, as the low bits of a selector byte: byte 3 of x >> 6 is x >> 30, byte 1 the
    // bits 15, 14, bytes 2 and 0 the bits 23, 22 and 7, 6 (under two more bits, masked away).  The selected table
    // byte holds the code in its upper nibble.
    constexpr uint32_t sel_mask = PK == 1 ? 0xFFFFFFFFu : PK == 2 ? 0x03000300u : 0x03030303u;
    constexpr uint32_t keep = PK == 1 ? 0x0FFFFFFFu : PK == 2 ? 0x0FFF0FFFu : 0x0F0F0F0Fu;
    uint32_t sel = x >> 6;
    if constexpr (PK > 1) sel &= sel_mask;
    const uint32_t top = __builtin_amdgcn_perm(0u, 0x90A01000u, sel);
    return make_uint2(e, (o & keep) | (top & ~keep));
}

// PK values of 32 / PK bits (two's complement, already clamped to that range) in one word, value p in bits
// 32 p / PK and up
template <int PK>
__device__ __forceinline__ uint32_t pack_values(const uint32_t (&v)[PK])
{
    if constexpr (PK == 1) {
        return v[0];
    } else if constexpr (PK == 2) {
        return __builtin_amdgcn_perm(v[1], v[0], 0x05040100u);       // bytes a0 a1 b0 b1
    } else {
        const uint32_t ab = __builtin_amdgcn_perm(v[1], v[0], 0x0C0C0400u);   // bytes a0 b0 0 0
        const uint32_t cd = __builtin_amdgcn_perm(v[3], v[2], 0x0C0C0400u);
        return __builtin_amdgcn_perm(cd, ab, 0x05040100u);
    }
}

// The 16 x 16 transpose of 4-bit elements that the LDS performs on a read (DS_READ_B64_TR_B4): in every group of
// 16 lanes, lane i receives nibble i of the 64-bit rows that the lanes e = 0 .. 15 of its group address, the one
// of lane e in nibble e.
typedef int v2i __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint2 lds_read_transposed(const uint2 *row)
{
    const v2i r = __builtin_amdgcn_ds_read_tr4_b64_v2i32((v2i __attribute__((address_space(3))) *)(row));
    return make_uint2((uint32_t)r.x, (uint32_t)r.y);
}

// Staging area of one wave for one chunk of 512 columns: 16 words x 32 columns x 8 bytes (the codes of a column).
// The row of column 4 n + r of word w sits at w * 40 + 8 r + n (in units of 8 bytes): the columns of one operand
// register are contiguous; a word takes 320 bytes, so that the 64-byte pieces that the lanes of a write put into
// adjacent words fall into different banks, and every position of a lane is a constant away from its first.
constexpr int kStageRows = 16 * 40;
// LDS integers of the kernels that cover wide rows in several passes (96 KB: with the staging areas of eight waves a
// workgroup stays below the 160 KB of a compute unit)
constexpr int kSplitInts = 24576;
__device__ __forceinline__ int stage_row(int w, int r, int n) { return w * 40 + 8 * r + n; }

// The same operand from the two plane words (bit c = column c) of a digit row: p0 the lower plane, p1 the upper
__device__ __forceinline__ void digit_operand_from_planes(uint32_t p0, uint32_t p1, u32x4 &dst)
{
    // digits of the even columns c at bits c, c + 1; of the odd columns c at bits c - 1, c
    uint32_t e = (p0 & 0x55555555u) | ((p1 << 1) & ~0x55555555u);
    uint32_t o = ((p0 >> 1) & 0x55555555u) | (p1 & ~0x55555555u);
    asm("" : "+v"(e), "+v"(o));   // (keeps the two words whole: ten operations instead of fourteen)
    dst.x = e & 0x33333333u;
    dst.y = o & 0x33333333u;
    dst.z = (e >> 2) & 0x33333333u;
    dst.w = (o >> 2) & 0x33333333u;
}

// digits (b1 b0) of the top row -> the codes of their signed value -2 b1 + b0; `top` = 0x22222222 in the lanes
// of digit 15, else 0 (then nothing changes)
__device__ __forceinline__ uint32_t signed_top_digit(uint32_t d, uint32_t top)
{
    return (d & ~((d << 1) & top)) | ((d & top) << 2);
}

__device__ __forceinline__ v8i as_operand(const u32x4 v)
{
    v8i r = {(int)v.x, (int)v.y, (int)v.z, (int)v.w, 0, 0, 0, 0};   // FP4 operands use the first four registers
    return r;
}

// One packed word -> the B operand: FP4 code 2.0 where the weight bit is set
__device__ __forceinline__ v8i weight_operand(uint32_t w)
{
    v8i r = {(int)((w << 2) & 0x44444444u), (int)((w << 1) & 0x44444444u), (int)(w & 0x44444444u),
             (int)((w >> 1) & 0x44444444u), 0, 0, 0, 0};
    return r;
}

// Two packed words (the same columns of two bitlayers) -> the B operand of their digits 2 hi + lo (FP4 code = digit)
__device__ __forceinline__ v8i weight_digit_operand(uint32_t hi, uint32_t lo)
{
    u32x4 d;
    digit_operand_from_planes(lo, hi, d);
    return as_operand(d);
}

// cbsz = blgp = 4: both operands FP4 (E2M1).  `scale_a`, `scale_b` are the E8M0 block scales of the operands: 127 =
// 2^0 on both sides for a weight operand of codes 2.0 (product = digit / 2 * 2), 128 = 2^1 on both sides for a weight
// operand of digits (product = 2 digit / 2 * 2 digit / 2 = digit * digit), so that the sums are the integers
// themselves; 128 + e on the weight side multiplies the products of one instruction by 2^e.
__device__ __forceinline__ v4f mfma_fp4(const v8i a, const v8i b, const v4f c, int scale_a, int scale_b)
{
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 4, 4, 0, scale_a, 0, scale_b);
}

// NQ: chunks of 512 columns per wave; NV: activation vectors whose digit rows a wave keeps (each weight block is
// expanded once and multiplied with all of them); MAXS: most waves (column slices) per workgroup, which bounds
// the registers a wave may use; RU: units (row tile, bitlayer pair) whose blocks a wave has in flight.  The host picks
// RU <= the units a wave has, so that a short stream pays for no empty ring slots; 4 KB in flight per wave
// measured best (more requests in flight than that slow the short streams down and do not speed up the long ones).
// PAIR: a unit is a pair of bitlayers (worth it when several vectors share the expanded weights; with one vector
// it measured 5-10 % slower up to 8192 columns and the same beyond: the stream starts later and a call has too few
// units for the saved instructions to show).
// PK: activation vectors per A operand.  With at most 16 (8) activation bits a vector has 8 (4) digits, the rest is
// sign extension, so 2 (4) vectors share the sixteen rows of an operand and one instruction serves them all
// (Section 3.1: fewer activation bits, less work).  NV then counts operands; a wave serves NV * PK vectors.
// IL: the packed words hold the digits of the bitlayer pairs already (PB_LAYOUT_TILE16_PAIRS_V1: even columns of a word
// in the block of the upper bitlayer, odd columns in the block of the lower one, sign bitlayer complemented): six
// operations per word pair instead of ten and no complement; a unit always reads both blocks, and a last single
// bitlayer is its pair's digit without the low bit.
// SPLIT: the columns of a row are covered in several passes, each with the waves' digit rows of its own range of
// MAXS * NQ chunks at most, over the same row tiles; a row tile's sums stay in LDS (one buffer per row tile of the
// round, as many row tiles per round as fit) and the last pass finishes it.  For batches on rows wider than the
// registers of a workgroup hold digit rows of four operands for: each expanded weight word then still serves four
// operands, at the price of rebuilding the digit rows once per pass and round.
template <int NQ, int NV, int MAXS, int RU, bool PAIR, int PK, bool IL = false, bool SPLIT = false>
__global__ __launch_bounds__(MAXS * 64) void k_mfma(const uint32_t *packed, const float *X0, uint32_t packed_bytes,
                                                    uint32_t flags, int cols0, int batch, uint32_t layer_step,
                                                    uint32_t round_step, int rounds_per_wg, int rt_count, int cq,
                                                    int m_used, const MfmaArgs a)
{
    const MfmaHead h = {packed, X0, packed_bytes, flags, cols0, batch, layer_step, round_step, rounds_per_wg, rt_count, cq, m_used};
    // Units requested before the activations have arrived (a head start that keeps HBM busy during the transpose);
    // the rest of the ring follows once the digit rows are built.
    // (two units measured best: with three or four a call of 4096 or 8192 columns takes 0.2-0.5 us longer)
    constexpr int PRE = NQ >= 4 ? 1 : (RU < 2 ? RU : 2);
    static_assert(PK == 1 || PAIR, "packed vectors run on the pair kernels");
    static_assert(!IL || PAIR, "the digit layout is read by the pair kernels");
    static_assert(!SPLIT || PAIR, "the kernels that split the columns are pair kernels");
    // sums per operand, bitlayer (or pair), row and kind of lane: the four operand rows of a lane of the result are
    // the even digits 0-6, the even digits 8-14, the odd digits 1-7, the odd digits 9-15 of one vector (PK = 1); the
    // even and the odd digits of two vectors (PK = 2: lanes kb = 0, 2 the first, kb = 1, 3 the second); with PK = 4 a
    // lane holds two digits of each of two vectors and keeps two sums.  The 64 lanes of a wave add to different
    // words.  Two buffers, used by alternate row tiles.  (The group sums of merged pairs live in the same memory
    // as [group][row][8 words] per buffer and operand: at most PB_MAX_BITS / 2 groups, which fits for every QN.)
    constexpr int QN = PK == 4 ? 8 : 4;
    static_assert(PB_MAX_BITS * QN >= (PB_MAX_BITS / 2) * 8, "room for the group sums");
    // (SPLIT: one buffer per row tile of a pass, see below, in `sbuf`)
    __shared__ __align__(16) int abuf[SPLIT ? 1 : 2][SPLIT ? 1 : NV][SPLIT ? 1 : PB_MAX_BITS][kTileRows][QN];
    __shared__ __align__(16) int sbuf[SPLIT ? kSplitInts : 4];
    __shared__ float s_scales[PB_MAX_BITS];
    // merged pairs: what the sign pair's digits count too much, per operand and kind of sum (see below)
    __shared__ __align__(16) int s_sx[NV][8];
    // staging area of the activation transpose, kStageRows rows of 8 bytes per wave (none when the planes are given)
    extern __shared__ __align__(16) unsigned char stage_lds[];

    const int lane_id = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // SPLIT: `parts` passes over the columns, each of cq_part chunks (every wave has the same slice in every pass,
    // a wave of the last pass maybe none); the loop below runs pass after pass, round after round.
    const int parts = SPLIT ? split_parts(h.cq, MAXS * NQ) : 1;
    const int cq_part = SPLIT ? split_chunks_per_part(h.cq, MAXS * NQ) : h.cq;   // chunks per pass
    const int nwaves = (cq_part + NQ - 1) / NQ;                 // = blockDim.x / 64 (the launcher's S), from a preloaded argument
    const int n0 = blockIdx.y * NV * PK;                        // first activation vector of this workgroup
    const int m = h.m;
    const int rt_first = blockIdx.x * h.rounds_per_wg;
    const int rounds_all = min(h.rounds_per_wg, h.rt_count - rt_first);  // >= 1 by construction
    // units of a row tile: the pairs (0, 1), (2, 3), ..., and a last single bitlayer if m is odd
    const int mp = PAIR ? (m + 1) / 2 : m;
    int turn = 0;         // (row tiles finished * RW) % nwaves, kept up by additions: the wave whose turn it is to finish a row tile
  for (int rt_base = 0, part = 0;;) {
    // (SPLIT: the lane number is taken anew in every pass, so that what a pass derives from it is worked out again
    // instead of occupying registers through the products of the pass before)
    int lane = lane_id;
    if constexpr (SPLIT) asm volatile("" : "+v"(lane));
    const int q0 = (part * nwaves + wave) * NQ;                 // first chunk of this wave's column slice
    const int nq = min(NQ, h.cq - q0);                          // chunks it really has (>= 1 by construction; SPLIT: maybe none)
    const int rt0 = rt_first + rt_base;
    // (SPLIT: row tiles of this pass: until the scales are known, a number that has room in either case; the first
    // requests of the ring, all that happens until then, do not depend on which)
    int rounds = SPLIT ? min(rounds_all - rt_base, kSplitInts / (NV * PB_MAX_BITS * kTileRows * QN)) : rounds_all;
    int U = rounds * mp;

    // layer scales, lane i holds scales[i] (and the next one, for the check of the pairs): requested after the
    // first weights (nothing that a wave requests before them may depend on the argument structure, which is still
    // on its way when a wave starts); parked in LDS once the digit rows are built (the barrier before the first final
    // sum orders that store)
    // (Buffer loads whose range ends after m scales, none without scales: no branch, so that the compiler's count of
    // the loads in flight stays exact and a wait for the activations does not turn into a wait for the weights.)
    float scv = 0.0f, scn = 0.0f;
    auto request_scales = [&]() {
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float *>(a.scales), 0, a.scales ? m * 4 : 0, 0x00020000);
        scv = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, lane * 4, 0, 0));
        if constexpr (PAIR) scn = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, lane * 4 + 4, 0, 0));
    };

    // ---- the weight stream of this wave: unit u = (round r, pair p): NQ blocks of 1 KB of the pair's low bitlayer
    // (2 p + 1, or the single one) and NQ of its high bitlayer (2 p, if the unit is a pair) ----
    const size_t base_off = (size_t)rt0 * h.round_step + (size_t)q0 * 1024;
    const char *base = reinterpret_cast<const char *>(h.packed) + base_off;
    const uint32_t avail = (uint32_t)(h.packed_bytes - base_off);
    const int voff = lane * 16;
    constexpr int SB = PAIR ? 2 * NQ : NQ;   // blocks of a unit
    // Cache policy of the weight loads: streaming (non-temporal) where a call reads every block once; the pair
    // kernels with four and more operands serve batches, whose vector groups read the same blocks at about the same
    // time on one XCD and should find them in its L2.  (Pair kernels with one or two operands run as a single
    // group: streaming measured 20 % faster there with two vectors.)
    constexpr int kWeightPolicy = (PAIR && NV > 2) ? 0 : 2;
    u32x4 ring[RU][SB];
    uint32_t ld_round = 0;
    int ld_p = 0, ld_u = 0;
    auto issue = [&](u32x4 (&dst)[SB]) {
        // past the last unit, and for chunks beyond the end of a ragged last slice, the descriptor has 0 records:
        // every lane is out of range, the load returns 0 and moves no data (no branch, so the compiler counts
        // the loads in flight exactly)
        const int lo_layer = !PAIR ? ld_p : (IL ? 2 * ld_p + 1 : min(2 * ld_p + 1, m - 1));
        const bool has_hi = PAIR && (IL || 2 * ld_p + 1 <= m - 1);
        const uint32_t lo_off = ld_round + (uint32_t)lo_layer * h.layer_step;
        const uint32_t hi_off = has_hi ? lo_off - h.layer_step : lo_off;
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<char *>(base), 0, (ld_u < U && q < nq) ? (int)avail : 0, 0x00020000);
            dst[q] = __builtin_amdgcn_raw_buffer_load_b128(rs, voff + q * 1024, (int)lo_off, kWeightPolicy);
        }
        if constexpr (PAIR) {
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
                    const_cast<char *>(base), 0, (ld_u < U && has_hi && q < nq) ? (int)avail : 0, 0x00020000);
                dst[NQ + q] = __builtin_amdgcn_raw_buffer_load_b128(rs, voff + q * 1024, (int)hi_off, kWeightPolicy);
            }
        }
        __builtin_amdgcn_sched_barrier(0x7);
        ++ld_u;
        if (++ld_p == mp) { ld_p = 0; ld_round += h.round_step; }
    };

    // LDS sums start at zero.  The barrier that orders this is taken after every wave has REQUESTED its activations
    // and before any wave requests weights: the memory pipeline of a CU returns data in request order, so an
    // activation load queued behind another wave's weight loads (HBM misses) would arrive a memory latency late.
    auto zero_sums_and_meet = [&]() {
        if constexpr (SPLIT) {
            // (later passes find the sums of the passes before them, or the zeros that the final sums left)
            if (rt_base == 0 && part == 0) {
                for (int i = threadIdx.x; i < kSplitInts; i += nwaves * 64) sbuf[i] = 0;
                if (threadIdx.x < NV * 8) (&s_sx[0][0])[threadIdx.x] = 0;
            }
        } else {
            for (int i = threadIdx.x; i < 2 * NV * PB_MAX_BITS * QN * kTileRows; i += nwaves * 64)
                (&abuf[0][0][0][0][0])[i] = 0;
            if (threadIdx.x < NV * 8) (&s_sx[0][0])[threadIdx.x] = 0;
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- the digit rows of this wave's slice, as A operands, kept in registers ----
    // lane l = 16 * kb + i: digit i (planes 2 i, 2 i + 1 of x_q) of the words 16 * q + 4 * kb + t
    const int kb = lane >> 4;
    u32x4 pa[NV][NQ][4];
    constexpr int VG = NV > 4 ? 4 : NV;   // vectors whose activations are in flight together
    if (PK == 1 && (h.flags & kPlanesGiven)) {
        const uint32_t top = (lane & 15) == 15 ? 0x22222222u : 0u;
#pragma unroll
        for (int g = 0; g < NV; g += VG) {
            uint4 pl0[VG][NQ], pl1[VG][NQ];
#pragma unroll
            for (int v = 0; v < VG; ++v) {
                const int n = min(n0 + g + v, h.batch - 1);
                const bool live = n0 + g + v < h.batch;
                const uint32_t *pl =
                    a.planes + ((size_t)n * 32 + 2 * digit_of_row(lane & 15)) * (size_t)a.cwp + (size_t)q0 * 16 + 4 * kb;
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    pl0[v][q] = pl1[v][q] = make_uint4(0, 0, 0, 0);
                    if (q < nq && live) {
                        pl0[v][q] = *reinterpret_cast<const uint4 *>(pl + q * 16);
                        pl1[v][q] = *reinterpret_cast<const uint4 *>(pl + (size_t)a.cwp + q * 16);
                    }
                }
            }
            if (g == 0) {
                zero_sums_and_meet();
#pragma unroll
                for (int k = 0; k < PRE; ++k) issue(ring[k]);
                request_scales();
            }
#pragma unroll
            for (int v = 0; v < VG; ++v)
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    const uint4 p0 = pl0[v][q], p1 = pl1[v][q];
                    digit_operand_from_planes(p0.x, p1.x, pa[g + v][q][0]);
                    digit_operand_from_planes(p0.y, p1.y, pa[g + v][q][1]);
                    digit_operand_from_planes(p0.z, p1.z, pa[g + v][q][2]);
                    digit_operand_from_planes(p0.w, p1.w, pa[g + v][q][3]);
#pragma unroll
                    for (int t = 0; t < 4; ++t)
#pragma unroll
                        for (int r = 0; r < 4; ++r) pa[g + v][q][t][r] = signed_top_digit(pa[g + v][q][t][r], top);
                }
        }
    } else {
        // Algorithm 2: x_q = Int(x * 2^f); then the transpose of Section 3.4 through LDS.  Lane L loads the
        // columns 256 j + 4 L .. + 3 (j = 0, 1) of a chunk with one 16-byte load each, converts them, writes the
        // sixteen digit codes of every column as one 8-byte row into this wave's staging area and reads the rows back
        // transposed: lane (kb, i) receives digit row i of the 32 columns of word 4 kb + t, register r = the
        // columns 4 n + r, which is the A operand as it stands.
        // Buffer loads return 0 beyond the end of a vector (checked dword by dword), and for the vectors beyond the
        // end of the batch.
        uint2 *stage = reinterpret_cast<uint2 *>(stage_lds) + wave * kStageRows;
        uint2 *const wr_row = stage + stage_row(lane >> 3, 0, lane & 7);   // a load's four columns: word 8 j + (lane >> 3), n = lane & 7
        const uint2 *const rd_row = stage + stage_row(4 * kb, (lane >> 3) & 1, lane & 7);
        const int col0 = 512 * q0 + 4 * lane;                 // first column of the lane's load j = 0 of chunk 0
        // operands whose activations are in flight together (PK vectors each)
        constexpr int VGP = PK >= VG ? 1 : VG / PK;
#pragma unroll
        for (int g = 0; g < NV; g += VGP) {
            u32x4 xv[VGP][PK][NQ][2];
#pragma unroll
            for (int v = 0; v < VGP; ++v)
#pragma unroll
                for (int p = 0; p < PK; ++p) {
                    const int nn = n0 + (g + v) * PK + p;
                    const int n = min(nn, h.batch - 1);
                    const bool live = nn < h.batch;
                    const __amdgpu_buffer_rsrc_t rx0 = __builtin_amdgcn_make_buffer_rsrc(
                        const_cast<float *>(h.X0 + (size_t)n * h.cols0), 0, live ? h.cols0 * 4 : 0, 0x00020000);
#pragma unroll
                    for (int q = 0; q < NQ; ++q)
#pragma unroll
                        for (int j = 0; j < 2; ++j)
                            xv[v][p][q][j] =
                                __builtin_amdgcn_raw_buffer_load_b128(rx0, (col0 + 512 * q + 256 * j) * 4, 0, 0);
                }
            // Second part of a concatenated input [X0 ; X1].  Offsets of columns that belong to the first part
            // would be negative: they are clamped and the value dropped (a negative register offset that an
            // instruction offset brings back above zero is not range-checked lane by lane on this hardware).
            // If cols0 is a multiple of 4 a lane's four columns lie in one part and one 16-byte load serves;
            // else every column is loaded by itself.
            u32x4 xw[VGP][PK][NQ][2];
            if (h.flags & kSecondPart) {
#pragma unroll
                for (int v = 0; v < VGP; ++v)
#pragma unroll
                    for (int p = 0; p < PK; ++p) {
                        const int nn = n0 + (g + v) * PK + p;
                        const int n = min(nn, h.batch - 1);
                        const bool live = nn < h.batch;
                        const __amdgpu_buffer_rsrc_t rx1 = __builtin_amdgcn_make_buffer_rsrc(
                            const_cast<float *>(a.X1 + (size_t)n * a.cols1), 0, live ? a.cols1 * 4 : 0, 0x00020000);
#pragma unroll
                        for (int q = 0; q < NQ; ++q)
#pragma unroll
                            for (int j = 0; j < 2; ++j) {
                                const int c1 = col0 + 512 * q + 256 * j - h.cols0;
                                if ((h.cols0 & 3) == 0) {
                                    xw[v][p][q][j] = __builtin_amdgcn_raw_buffer_load_b128(rx1, max(c1, 0) * 4, 0, 0);
                                } else {
#pragma unroll
                                    for (int r = 0; r < 4; ++r)
                                        xw[v][p][q][j][r] =
                                            __builtin_amdgcn_raw_buffer_load_b32(rx1, max(c1 + r, 0) * 4, 0, 0);
                                }
                            }
                    }
            }
            if (g == 0) {
                zero_sums_and_meet();
#pragma unroll
                for (int k = 0; k < PRE; ++k) issue(ring[k]);
                request_scales();
            }
            if (h.flags & kSecondPart) {
#pragma unroll
                for (int v = 0; v < VGP; ++v)
#pragma unroll
                    for (int p = 0; p < PK; ++p)
#pragma unroll
                        for (int q = 0; q < NQ; ++q)
#pragma unroll
                            for (int j = 0; j < 2; ++j)
#pragma unroll
                                for (int r = 0; r < 4; ++r)
                                    xv[v][p][q][j][r] |=
                                        col0 + 512 * q + 256 * j + r >= h.cols0 ? xw[v][p][q][j][r] : 0u;
            }
#pragma unroll
            for (int v = 0; v < VGP; ++v)
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    // (the reads of the chunk before have returned: their registers were waited for below)
                    // (32-bit activations need no clamp after the conversion: one instruction less per value)
                    auto write_rows = [&](auto narrow) {
#pragma unroll
                        for (int j = 0; j < 2; ++j)
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                uint32_t xq[PK];
#pragma unroll
                                for (int p = 0; p < PK; ++p)
                                    xq[p] = (uint32_t)to_fixed_point<decltype(narrow)::value>(
                                        __uint_as_float(xv[v][p][q][j][r]), a.fscale, a.imin, a.imax);
                                wr_row[stage_row(8 * j, r, 0)] = digit_codes<PK>(pack_values<PK>(xq));
                            }
                    };
                    if (PK > 1 || a.imin != INT32_MIN) write_rows(std::true_type{});
                    else write_rows(std::false_type{});
                    // the wave's own writes have landed before its lanes read each other's rows
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const uint2 lo = lds_read_transposed(rd_row + stage_row(t, 0, 0));
                        const uint2 hi = lds_read_transposed(rd_row + stage_row(t, 2, 0));
                        pa[g + v][q][t] = u32x4{lo.x, lo.y, hi.x, hi.y};
                    }
                    // ... and the reads have returned before the next chunk overwrites the rows
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    __builtin_amdgcn_wave_barrier();
                }
        }
    }
    if (wave == 0 && lane < PB_MAX_BITS) s_scales[lane] = scv;
    // Pairs are merged if every scale is half the one before, minus half for the one after the sign bitlayer (then
    // s_hi A_hi + s_lo A_lo = s_lo (+-2 A_hi + A_lo), and the pairs of a row tile are in the ratio 4 to each other)
    bool merged = PAIR && a.pairs_out != 0;
    if (PAIR && !a.A) {
        const bool off = lane + 1 < m && !(scv == (lane == 0 ? -2.0f : 2.0f) * scn);
        merged = __builtin_amdgcn_ballot_w64(off) == 0;
    }
    // (With the sums of the pairs asked for, a group is one pair.)
    const int gsize = a.pairs_out ? 1 : kPairGroup;
    const int nsets = merged ? (mp + gsize - 1) / gsize : m;   // sets of sums of a row tile and operand
    // SPLIT: the sums of a row tile are NV * set_ints integers, row tile after row tile (group sums take 8 integers
    // per row; bitlayer by bitlayer every operand has room for all PB_MAX_BITS sets, which the final sum may read)
    const int set_ints = merged ? nsets * (kTileRows * 8) : PB_MAX_BITS * kTileRows * QN;
    if constexpr (SPLIT) {
        const int left = rounds_all - rt_base, cap = kSplitInts / (NV * set_ints);
        const int passes = (left + cap - 1) / cap;
        rounds = (left + passes - 1) / passes;   // (even shares)
        U = rounds * mp;
    }
    __builtin_amdgcn_sched_barrier(0);   // the rest of the ring is requested after the activations have arrived
#pragma unroll
    for (int k = PRE; k < RU; ++k) issue(ring[k]);

    // The four registers of a lane of the result are the operand rows 4 kb + c: the digits b, b + 2, b + 4, b + 6
    // with b = 0, 8, 1, 9 for kb = 0 .. 3.  A lane adds them up with the weights 16^c (in units of 4^b) and the sums
    // of the four kinds of lanes stay apart until the row tile is finished.
    // Bitlayer by bitlayer: sums of digit products are <= 9 * 2048 (a slice has at most 2048 columns): c0 + 16 c1 and
    // c2 + 16 c3 are exact in fp32 (< 2^19), their combination is an integer below 2^27.
    // With PK = 2 the same four registers are four digits (even or odd) of one of two vectors; with PK = 4 two
    // digits of each of two vectors, and the lane keeps the two halves c0 + 16 c1, c2 + 16 c3 apart.
    constexpr int LS = PK == 4 ? 2 : 1;   // sums of a lane per operand
    auto lane_sums = [](const v4f acc, int (&out)[LS]) {
        const float t0 = fmaf(acc[1], 16.0f, acc[0]), t1 = fmaf(acc[3], 16.0f, acc[2]);
        if constexpr (PK == 4) {
            out[0] = (int)t0;
            out[1] = (int)t1;
        } else {
            out[0] = (int)t0 + ((int)t1 << 8);
        }
    };
    const int j = lane & 15;
    int pp = 0, pr = 0;   // pair and round of the unit being multiplied
    // the sums of operand v of the row tile being multiplied: two buffers used by alternate row tiles, or (SPLIT)
    // one per row tile of the pass
    auto sums_of = [&](int v) -> int * {
        if constexpr (SPLIT) return sbuf + (pr * NV + v) * set_ints;
        else return &abuf[pr & 1][v][0][0][0];
    };
    // the end of a bitlayer: the sums of this lane go to `set` in LDS
    auto finish = [&](const v4f (&acc)[NV], int set) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            int ls[LS];
            lane_sums(acc[v], ls);
#pragma unroll
            for (int e = 0; e < LS; ++e) atomicAdd(sums_of(v) + (set * kTileRows + j) * QN + LS * kb + e, ls[e]);
        }
    };
    // Merged pairs: the pairs of a row tile accumulate in ONE set of registers.  With all scales halving, pair p
    // counts 2^e times the last pair of its group (e = the distance between their low bitlayers), and the block scale
    // of the weight operand supplies that factor: a group of up to kPairGroup pairs costs one conversion and one LDS
    // update instead of one per pair.  Bounds: a register holds at most 9 * 2048 * (1 + 4 + .. + 4^4) = 6.3 M < 2^24
    // (exact in fp32); the two halves c0 + 16 c1 and c2 + 16 c3 of a lane are integers of their own in LDS, over the
    // slices of a row at most 17 * 9 * 32768 * 341 = 1.71e9 < 2^31.
    // low bitlayer of a unit of a pair kernel (IL: of the pair as stored, which a last single bitlayer has without
    // using it: bitlayer m, with half the scale of bitlayer m - 1, minus half if that is the sign bitlayer)
    auto low_layer = [&](int unit) { return IL ? 2 * unit + 1 : min(2 * unit + 1, m - 1); };
    auto layer_scale = [&](int layer) {
        return layer < m ? s_scales[layer] : (m == 1 ? -0.5f : 0.5f) * s_scales[m - 1];
    };
    // sum_c x_q[c] over the slice, in the form of the group sums: the product with an operand of digits 1, doubled
    // (the digits of the sign pair stand 2 too high in every column) and with the factor of pair 0 in its group.
    // It is the same for every row: the slices add theirs up in LDS once per call (SPLIT: every pass of the first
    // round its columns') and the final sum takes it off the first group of every row.
    if (PAIR && merged && (IL || m >= 2) && (!SPLIT || rt_base == 0)) {
        const v8i ones = {0x11111111, 0x11111111, 0x11111111, 0x11111111, 0, 0, 0, 0};
        const int e0 = low_layer(min(gsize, mp) - 1) - 1 + 1;   // (+ 1: doubled)
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            v4f acc = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int q = 0; q < NQ; ++q)
#pragma unroll
                for (int t = 0; t < 4; ++t) acc = mfma_fp4(as_operand(pa[v][q][t]), ones, acc, 128, 128);
            int s0 = ((int)acc[0] + ((int)acc[1] << 4)) << e0, s1 = ((int)acc[2] + ((int)acc[3] << 4)) << e0;
            // (the matrix instructions need every lane: the sums are pinned here so that the compiler does not move
            // their computation into the branch of the lanes that add them up, as it did)
            asm volatile("" : "+v"(s0), "+v"(s1));
            if (j == 0) {
                atomicAdd(&s_sx[v][2 * kb], s0);
                atomicAdd(&s_sx[v][2 * kb + 1], s1);
            }
        }
    }
    v4f accg[NV];         // the sums of the group being multiplied
    int gfirst = 0, gset = 0;   // its first pair, its index in the row tile
    // the end of a group: its sums go to LDS, eight integers per (operand, group, row): word 2 kb + e is the half e
    // of the lanes of kind kb
    auto finish_group = [&]() {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int i0 = (int)accg[v][0] + ((int)accg[v][1] << 4);
            const int i1 = (int)accg[v][2] + ((int)accg[v][3] << 4);
            int *dst = sums_of(v) + gset * (kTileRows * 8) + j * 8 + 2 * kb;
            atomicAdd(dst, i0);
            atomicAdd(dst + 1, i1);
        }
    };
    for (int u0 = 0; u0 < U; u0 += RU) {
#pragma unroll
        for (int k = 0; k < RU; ++k) {
            if (u0 + k < U) {
                const int lo_layer = !PAIR ? pp : (IL ? 2 * pp + 1 : min(2 * pp + 1, m - 1));
                const bool has_hi = PAIR && (IL || 2 * pp + 1 <= m - 1);
                // (chunks beyond a ragged last slice, and the absent high bitlayer of a single unit, are zero words)
                if (PAIR && merged) {
                    if (pp == gfirst) {
#pragma unroll
                        for (int v = 0; v < NV; ++v) accg[v] = v4f{0.f, 0.f, 0.f, 0.f};
                    }
                    const int glast = min(gfirst + gsize, mp) - 1;             // last pair of this group
                    const int bscale = 128 + low_layer(glast) - lo_layer;     // 2^1 for the digits, 2^e for the pair
                    const bool sign_pair = pp == 0 && has_hi;
                    const uint32_t inv = (!IL && sign_pair) ? 0xFFFFFFFFu : 0u;   // the sign bitlayer enters as 1 - w
                    // (IL) a last single bitlayer: the digits without their low bits
                    const uint32_t dmask = (IL && 2 * pp + 1 >= m) ? 0x22222222u : 0x33333333u;
#pragma unroll
                    for (int q = 0; q < NQ; ++q) {
                        const u32x4 wl = ring[k][q];
                        u32x4 wh = ring[k][PAIR ? NQ + q : q];
                        if constexpr (!IL) wh ^= inv;
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            v8i b;
                            if constexpr (IL) {   // wh: digits of the even columns, wl: of the odd columns
                                b = v8i{(int)(wh[t] & dmask), (int)(wl[t] & dmask), (int)((wh[t] >> 2) & dmask),
                                        (int)((wl[t] >> 2) & dmask), 0, 0, 0, 0};
                            } else {
                                b = weight_digit_operand(wh[t], wl[t]);
                            }
#pragma unroll
                            for (int v = 0; v < NV; ++v)
                                accg[v] = mfma_fp4(as_operand(pa[v][q][t]), b, accg[v], 128, bscale);
                        }
                    }
                    if (pp == glast) {
                        finish_group();
                        gfirst += gsize;
                        ++gset;
                    }
                } else {
#pragma unroll
                    for (int h = PAIR ? 1 : 0; h >= 0; --h) {
                        if (h == 1 && !has_hi) continue;
                        if (IL && h == 0 && 2 * pp + 1 >= m) continue;   // (the pair's lower bitlayer is not asked for)
                        v4f acc[NV];
#pragma unroll
                        for (int v = 0; v < NV; ++v) acc[v] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int q = 0; q < NQ; ++q) {
                            u32x4 w = ring[k][h * NQ + q];
                            if constexpr (IL) {   // the bits of one bitlayer out of the digit words
                                const u32x4 ev = ring[k][NQ + q], od = ring[k][q];
#pragma unroll
                                for (int t = 0; t < 4; ++t) {
                                    uint32_t upper, lower;
                                    pair_of_digits(ev[t], od[t], &upper, &lower);
                                    w[t] = h == 0 ? lower : (pp == 0 ? ~upper : upper);
                                }
                            }
#pragma unroll
                            for (int t = 0; t < 4; ++t) {
                                const v8i b = weight_operand(w[t]);
#pragma unroll
                                for (int v = 0; v < NV; ++v) acc[v] = mfma_fp4(as_operand(pa[v][q][t]), b, acc[v], 127, 127);
                            }
                        }
                        finish(acc, lo_layer - h);
                    }
                }
                if (++pp == mp) {
                    // The row tile is complete in every slice: scale and store it.  (The barrier per row tile also
                    // keeps the waves of a workgroup on one contiguous region of the weight stream; letting them
                    // drift apart over several row tiles measured 5-15 % slower.)
                    // A lane per (vector, row), or with one or two vectors per workgroup 4 or 2 lanes that share out the
                    // bitlayers: scaled sums in fp64, then the sum over those lanes (rows of 16 lanes 16 or 32 apart).
                    // The waves take turns, so that none of them is always late for the next barrier.
                    pp = 0;
                    gfirst = gset = 0;
                    __syncthreads();
                    constexpr int LG = NV >= 4 ? 1 : 4 / NV;            // lanes per operand and row
                    constexpr int RW = (NV * LG * kTileRows + 63) / 64; // waves that one row tile's outputs occupy
                    // (SPLIT: only the last pass over the columns finishes the row tiles)
                    for (int duty = (SPLIT && part + 1 < parts) ? RW : wave - turn + (wave < turn ? nwaves : 0); duty < RW;
                         duty += nwaves) {
                        const int slot = duty * 4 + (lane >> 4);
                        const int v = slot / LG, lg = slot % LG, jrow = lane & 15;
                        const int prow = (rt0 + pr) * kTileRows + jrow;
                        const int row = a.gate_h ? gates_matrix_row(prow, a.gate_h) : prow;
                        const bool row_ok = v < NV && row >= 0 && row < a.R;
                        int4 *src = reinterpret_cast<int4 *>(sums_of(v < NV ? v : 0) + (lg * kTileRows + jrow) * QN);
                        // bias and previous cell state of this lane's outputs: requested before the sums are read and
                        // added up, so that their way through memory is not waited for at the end (range-checked
                        // loads: 0 for absent arrays and for lanes without an output)
                        constexpr int kNoOutput = 0x7FFFFFF0;   // an offset beyond every array
                        const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(
                            const_cast<float *>(a.bias), 0, a.bias ? a.R * 4 : 0, 0x00020000);
                        const float bias_row =
                            __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rb, row_ok ? row * 4 : kNoOutput, 0, 0));
                        const __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc(
                            const_cast<float *>(a.c_prev), 0, a.c_prev ? h.batch * a.gate_h * 4 : 0, 0x00020000);
                        float c_old[PK];
#pragma unroll
                        for (int p = 0; p < PK; ++p) {
                            const int n = n0 + v * PK + p;
                            const bool cell = row_ok && n < h.batch && (lane & 3) == 0 && lg == 0;
                            c_old[p] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(
                                rc, cell ? (n * a.gate_h + row) * 4 : kNoOutput, 0, 0));
                        }
                        double z[PK];
#pragma unroll
                        for (int p = 0; p < PK; ++p) z[p] = 0.0;
                        if (PAIR && merged) {
                            // group sums: the halves (i0, i1) of the four kinds of lanes; Q_kb = i0 + 256 i1 is what a
                            // lane of kind kb would have had in one word
                            int *grp = sums_of(v < NV ? v : 0) + jrow * 8;
                            for (int g = lg; v < NV && g < nsets; g += LG) {
                                int4 *g4 = reinterpret_cast<int4 *>(grp + g * (kTileRows * 8));
                                const int4 t0 = g4[0], t1 = g4[1];
                                g4[0] = g4[1] = make_int4(0, 0, 0, 0);
                                int w[8] = {t0.x, t0.y, t0.z, t0.w, t1.x, t1.y, t1.z, t1.w};
                                if (g == 0) {   // the sign pair's group (zeros if there is nothing to take off)
                                    const int4 *sx4 = reinterpret_cast<const int4 *>(&s_sx[v < NV ? v : 0][0]);
                                    const int4 x0 = sx4[0], x1 = sx4[1];
                                    w[0] -= x0.x; w[1] -= x0.y; w[2] -= x0.z; w[3] -= x0.w;
                                    w[4] -= x1.x; w[5] -= x1.y; w[6] -= x1.z; w[7] -= x1.w;
                                }
                                // the group carries the scale of the low bitlayer of its last pair
                                const int si = low_layer(min((g + 1) * gsize, mp) - 1);
                                // (IL, sums of the pairs asked for) a single bitlayer came as twice itself, the sign
                                // bitlayer by itself as -2 A_0
                                const bool halve = IL && 2 * g + 1 >= m;
#pragma unroll
                                for (int p = 0; p < PK; ++p) {
                                    const int n = n0 + v * PK + p;
                                    if (a.A) {
                                        long long Q[4];
#pragma unroll
                                        for (int c = 0; c < 4; ++c) Q[c] = (long long)w[2 * c] + 256 * (long long)w[2 * c + 1];
                                        const long long sum = PK == 1   ? Q[0] + 4 * Q[2] + ((Q[1] + 4 * Q[3]) << 16)
                                                              : PK == 2 ? Q[p] + 4 * Q[2 + p]
                                                                        : (long long)w[p] + 4 * (long long)w[4 + p];
                                        if (row_ok && n < h.batch)
                                            a.A[((size_t)g * h.batch + n) * (size_t)a.R + row] =
                                                !halve ? sum : (g == 0 ? -sum : sum) / 2;
                                    } else {
                                        // (every part converts exactly; the last step rounds once if the sum is
                                        // beyond 2^53, as the conversion of the 64-bit integer would)
                                        double Q[4];
#pragma unroll
                                        for (int c = 0; c < 4; ++c) Q[c] = fma(256.0, (double)w[2 * c + 1], (double)w[2 * c]);
                                        const double sum = PK == 1   ? fma(65536.0, fma(4.0, Q[3], Q[1]), fma(4.0, Q[2], Q[0]))
                                                           : PK == 2 ? fma(4.0, Q[2 + p], Q[p])
                                                                     : fma(4.0, (double)w[4 + p], (double)w[p]);
                                        z[p] = fma((double)layer_scale(si), sum, z[p]);
                                    }
                                }
                            }
                        } else {
                            // PK = 1, the quarters of one vector: digits 0, 2, 4, 6 in units of 1, digits 8 .. 14 in units
                            // of 4^8, digits 1 .. 7 in units of 4, digits 9 .. 15 in units of 4^9; each below 2^31 in
                            // magnitude (4369 * 9 * 32768 columns).  PK = 2, 4: even digits + 4 * odd digits of vector p.
                            constexpr int SET = kTileRows * (QN / 4);   // int4s from one set of sums to the next
                            if (v < NV && a.A) {
                                for (int i = lg; i < nsets; i += LG, src += LG * SET) {
                                    int qv[QN];
#pragma unroll
                                    for (int e = 0; e < QN / 4; ++e) {
                                        const int4 t = src[e];
                                        src[e] = make_int4(0, 0, 0, 0);
                                        qv[4 * e] = t.x; qv[4 * e + 1] = t.y; qv[4 * e + 2] = t.z; qv[4 * e + 3] = t.w;
                                    }
#pragma unroll
                                    for (int p = 0; p < PK; ++p) {
                                        const long long sum =
                                            PK == 1 ? (long long)qv[0] + 4 * (long long)qv[2] +
                                                          (((long long)qv[1] + 4 * (long long)qv[3]) << 16)
                                                    : (long long)qv[p] + 4 * (long long)qv[PK + p];
                                        const int n = n0 + v * PK + p;
                                        if (row_ok && n < h.batch) a.A[((size_t)i * h.batch + n) * (size_t)a.R + row] = sum;
                                    }
                                }
                            } else if (v < NV) {
                                // The sets of a lane are read CH at a time, together with their scales, so that the LDS
                                // latency is paid once: sets beyond the last one hold zeros (nothing ever adds to them) and
                                // add nothing.  The 32-bit parts convert to fp64 exactly and so does their combination
                                // (below 2^51), which is the integer sum itself.
                                constexpr int MAXI = PB_MAX_BITS / LG;   // sets a lane can have
                                constexpr int CH = LG == 4 ? 2 : 4;      // (a chunk covers eight sets, or four)
                                static_assert(MAXI % CH == 0, "whole chunks");
                                for (int k0 = 0; k0 * LG < nsets; k0 += CH, src += CH * LG * SET) {
                                    int4 t[CH][QN / 4];
                                    float sc[CH];
#pragma unroll
                                    for (int c = 0; c < CH; ++c) {
                                        const int i = lg + LG * (k0 + c);          // < PB_MAX_BITS
#pragma unroll
                                        for (int e = 0; e < QN / 4; ++e) t[c][e] = src[c * LG * SET + e];
                                        // a merged pair carries the scale of its low bitlayer
                                        sc[c] = s_scales[!merged ? i : min(2 * i + 1, m - 1)];
                                    }
#pragma unroll
                                    for (int c = 0; c < CH; ++c)
#pragma unroll
                                        for (int e = 0; e < QN / 4; ++e) src[c * LG * SET + e] = make_int4(0, 0, 0, 0);
#pragma unroll
                                    for (int c = 0; c < CH; ++c) {
                                        double qd[QN];
#pragma unroll
                                        for (int e = 0; e < QN / 4; ++e) {
                                            qd[4 * e] = (double)t[c][e].x; qd[4 * e + 1] = (double)t[c][e].y;
                                            qd[4 * e + 2] = (double)t[c][e].z; qd[4 * e + 3] = (double)t[c][e].w;
                                        }
#pragma unroll
                                        for (int p = 0; p < PK; ++p) {
                                            const double sum = PK == 1 ? fma(65536.0, fma(4.0, qd[3], qd[1]), fma(4.0, qd[2], qd[0]))
                                                                       : fma(4.0, qd[PK + p], qd[p]);
                                            z[p] = fma((double)sc[c], sum, z[p]);
                                        }
                                    }
                                }
                            }
                        }
#pragma unroll
                        for (int p = 0; p < PK; ++p) {
                            if (LG >= 2) z[p] = add_across<16>(z[p]);
                            if (LG == 4) z[p] = add_across<32>(z[p]);
                        }
                        if (!a.A) {
#pragma unroll
                            for (int p = 0; p < PK; ++p) {
                                const int n = n0 + v * PK + p;
                                const bool live = row_ok && n < h.batch;
                                float y = (float)(z[p] * a.out_scale);
                                if (a.bias && live) y += bias_row;
                                if (a.c_prev) {
                                    // LSTM cell: the four lanes of a quad hold the gates i, f, g, o of one unit (row =
                                    // unit for gate i).  Every lane applies its own gate's nonlinearity (the logistic
                                    // function as 0.5 tanh(y / 2) + 0.5: one evaluation per lane, side by side), then
                                    // the first lane of the quad collects the four and updates the unit.
                                    const bool is_g = (lane & 3) == 2;
                                    const float th = tanhf(is_g ? y : 0.5f * y);
                                    const float act = is_g ? th : fmaf(0.5f, th, 0.5f);
                                    const float gi = __uint_as_float(dpp_mov<0x00>(__float_as_uint(act)));
                                    const float gf = __uint_as_float(dpp_mov<0x55>(__float_as_uint(act)));
                                    const float gg = __uint_as_float(dpp_mov<0xAA>(__float_as_uint(act)));
                                    const float go = __uint_as_float(dpp_mov<0xFF>(__float_as_uint(act)));
                                    const float cn = fmaf(gf, c_old[p], gi * gg);
                                    const float hn = go * tanhf(cn);
                                    if ((lane & 3) == 0 && live && lg == 0) {
                                        const size_t at = (size_t)n * a.gate_h + (size_t)row;
                                        a.c_out[at] = cn;
                                        a.h_out[at] = hn;
                                    }
                                } else {
                                    if (a.relu) y = fmaxf(y, 0.0f);
                                    if (live && lg == 0) a.Y[(size_t)n * a.R + row] = y;
                                }
                            }
                        }
                    }
                    ++pr;
                    turn += RW;
                    while (turn >= nwaves) turn -= nwaves;   // (RW <= 2: at most two rounds)
                }
            }
            issue(ring[k]);
        }
    }
    if constexpr (!SPLIT) break;
    if (++part == parts) {
        part = 0;
        rt_base += rounds;
        if (rt_base >= rounds_all) break;
    }
  }
}

// The kernel variants: (chunks per wave, operands per wave, most slices per workgroup, ring depth in units), each for
// single bitlayers, for pairs, for pairs with two and four vectors per operand, and the three pair kernels again for
// the layout that stores the digits of the pairs (fn[kind]; the variants with eight operands have no kind with four
// vectors per operand: their sums would not fit the LDS).
constexpr int kKinds = 7;
struct Variant {
    int nq, nv, maxs, ru;
    const void *fn[kKinds];
};
enum { kSingle = 0, kPairs = 1, kPairs2 = 2, kPairs4 = 3, kDigits = 3 };   // kind of the digit layout = kDigits + pair kind
// (pair kernels exist with rings of one and two units, see pick_ring; with four vectors per operand for at most four
// operands)
template <int NQ, int NV, int MAXS, int RU, int PK, bool IL>
static const void *pair_kernel()
{
    if constexpr (RU <= 2 && (PK < 4 || NV <= 4)) return reinterpret_cast<const void *>(k_mfma<NQ, NV, MAXS, RU, true, PK, IL>);
    else return nullptr;
}
#define PB_VARIANT(NQ, NV, MAXS, RU)                                                                \
    {NQ, NV, MAXS, RU, {reinterpret_cast<const void *>(k_mfma<NQ, NV, MAXS, RU, false, 1>),         \
                        pair_kernel<NQ, NV, MAXS, RU, 1, false>(), pair_kernel<NQ, NV, MAXS, RU, 2, false>(),  \
                        pair_kernel<NQ, NV, MAXS, RU, 4, false>(), pair_kernel<NQ, NV, MAXS, RU, 1, true>(),   \
                        pair_kernel<NQ, NV, MAXS, RU, 2, true>(), pair_kernel<NQ, NV, MAXS, RU, 4, true>()}}
static const Variant kVariants[] = {
    PB_VARIANT(1, 1, 16, 1), PB_VARIANT(1, 1, 16, 2), PB_VARIANT(1, 1, 16, 4),
    PB_VARIANT(1, 2, 16, 1), PB_VARIANT(1, 2, 16, 2), PB_VARIANT(1, 2, 16, 4),
    PB_VARIANT(1, 4, 8, 1),  PB_VARIANT(1, 4, 8, 2),  PB_VARIANT(1, 4, 8, 4),
    PB_VARIANT(1, 8, 8, 1),  PB_VARIANT(1, 8, 8, 2),  PB_VARIANT(1, 8, 8, 4),
    PB_VARIANT(2, 1, 16, 1), PB_VARIANT(2, 1, 16, 2), PB_VARIANT(2, 1, 16, 3),
    PB_VARIANT(2, 2, 8, 1),  PB_VARIANT(2, 2, 8, 2),
    PB_VARIANT(2, 4, 8, 1),  PB_VARIANT(2, 4, 8, 2),
    PB_VARIANT(4, 1, 8, 1),  PB_VARIANT(4, 1, 8, 2),
    PB_VARIANT(4, 1, 16, 1),
    PB_VARIANT(4, 2, 8, 1),  PB_VARIANT(4, 2, 8, 2),
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

// The kernels that cover wide rows in several passes, by kind (pair kernels only), in two shapes: two chunks and
// four operands per wave (passes of 8192 columns), one chunk and eight operands per wave (passes of 4096 columns);
// eight waves, two units in flight.  (With eight operands there is no kind with four vectors per operand: its sums
// would leave the LDS room for a single row tile per round.)
struct SplitShape {
    int nq, nv, chunks;
    const void *fn[kKinds];
};
constexpr int kSplitMaxS = 8;
#define PB_SPLIT(NQ, NV, PK, IL) reinterpret_cast<const void *>(k_mfma<NQ, NV, kSplitMaxS, 2, true, PK, IL, true>)
static const SplitShape kSplitShapes[2] = {
    {2, 4, kSplitChunks4, {nullptr, PB_SPLIT(2, 4, 1, false), PB_SPLIT(2, 4, 2, false), PB_SPLIT(2, 4, 4, false),
                           PB_SPLIT(2, 4, 1, true), PB_SPLIT(2, 4, 2, true), PB_SPLIT(2, 4, 4, true)}},
    {1, 8, kSplitChunks8, {nullptr, PB_SPLIT(1, 8, 1, false), PB_SPLIT(1, 8, 2, false), nullptr,
                           PB_SPLIT(1, 8, 1, true), PB_SPLIT(1, 8, 2, true), nullptr}},
};
static_assert(2 * kSplitMaxS == kSplitChunks4 && 1 * kSplitMaxS == kSplitChunks8, "the chunks of a pass are those of eight waves");

// Overrides of the launcher's choices (chunks and vectors per wave, ring depth, workgroups, pairs), for sweeps over
// the variants: compiled in only with -DPB_TUNING (a tuning build reads them from the environment once); the
// product build has none and its behaviour does not depend on the environment.  0 / -1 = not set.
struct Tuning {
    int nq = 0, nv = 0, ru = 0, wgs = 0, pair = -1, split = -1;
#ifdef PB_TUNING
    Tuning()
    {
        auto get = [](const char *name, int unset) { const char *e = getenv(name); return e ? atoi(e) : unset; };
        nq = get("PB_TUNE_NQ", 0); nv = get("PB_TUNE_NV", 0); ru = get("PB_TUNE_RU", 0);
        wgs = get("PB_TUNE_WGS", 0); pair = get("PB_TUNE_PAIR", -1); split = get("PB_TUNE_SPLIT", -1);
        if (nq < 0) nq = 0;
        if (nv < 0) nv = 0;
        if (ru < 0) ru = 0;
        if (wgs < 0) wgs = 0;
    }
#endif
};
static const Tuning &tuning()
{
    static const Tuning t;
    return t;
}

// As many vectors per wave as the batch has and the registers allow (each weight block is then read and expanded
// once for all of them), then the smallest slice (most waves per row, shortest transpose per wave) whose slice
// count fits a workgroup; ring depth 1 (the deeper rings are picked once the units per wave are known).
static int pick_variant(const Layout &L, int batch, int kind)
{
    const int want_nq = tuning().nq, want_nv = tuning().nv;
    int best = -1;
    for (int i = 0; i < kNumVariants; ++i) {
        const Variant &v = kVariants[i];
        if (v.ru != 1 || !v.fn[kind]) continue;
        if ((L.cq + v.nq - 1) / v.nq > v.maxs) continue;
        if (want_nq && v.nq != want_nq) continue;
        // no more than one empty half; eight operands only for more than sixteen (up to there groups of four, on more
        // workgroups, measured the same or up to 10 % faster; from 24 on eight are 14-18 % faster)
        if (want_nv ? v.nv != want_nv : ((v.nv > 1 && v.nv / 2 >= batch) || (v.nv == 8 && batch <= 16))) continue;
        if (best < 0 || v.nv > kVariants[best].nv || (v.nv == kVariants[best].nv && v.nq < kVariants[best].nq))
            best = i;
    }
    return best;
}

// The sibling of variant `vi` with the deepest ring that a wave with `units` units fills; with three units and
// rings of 2 and 4 to choose from, the deeper one (a wave with one or two units is faster without empty ring slots,
// one with three is 0.2 us faster when all three are in flight).  A unit of a pair kernel is two blocks per chunk:
// two units in flight are its best (four measured 4-13 % slower at 8192 columns and 17-21 % at 4096).
static int pick_ring(int vi, int units, int kind)
{
    const int want = tuning().ru;
    int best = vi;
    for (int i = 0; i < kNumVariants; ++i) {
        const Variant &v = kVariants[i];
        if (v.nq != kVariants[vi].nq || v.nv != kVariants[vi].nv || v.maxs != kVariants[vi].maxs || !v.fn[kind]) continue;
        const int cap = kind != kSingle ? (units < 2 ? units : 2) : (units == 3 ? 4 : units);
        if (want ? v.ru == want : (v.ru <= cap && v.ru > kVariants[best].ru)) best = i;
    }
    return best;
}

// Dynamic LDS of a workgroup of S waves: the staging area of the activation transpose.
static size_t stage_bytes(int S) { return (size_t)S * kStageRows * sizeof(uint2); }

// Workgroups of S waves that fit on the device at once (occupancy does not change while the process lives, so it
// is looked up once per kernel variant and workgroup size).
static int resident_workgroups(int variant, int S, int kind)
{
    static int cache[kKinds][kNumVariants][kMaxSlices + 1];
    int *slot = &cache[kind][variant][S];
    int v = __atomic_load_n(slot, __ATOMIC_RELAXED);
    if (v > 0) return v;
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    // (a workgroup's dynamic LDS may exceed the default limit of 64 KB, a compute unit of this chip has 160 KB:
    // declared for this variant and its siblings of other ring depths, one of which is the one launched)
    const void *fn = kVariants[variant].fn[kind];
    if (stage_bytes(S) > 32 * 1024) {
        for (int i = 0; i < kNumVariants; ++i) {
            const Variant &o = kVariants[i];
            if (o.nq != kVariants[variant].nq || o.nv != kVariants[variant].nv || o.maxs != kVariants[variant].maxs ||
                !o.fn[kind])
                continue;
            if (hipFuncSetAttribute(o.fn[kind], hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)stage_bytes(S)) != hipSuccess)
                return 0;
        }
    }
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(
            &per_cu, fn, S * 64, stage_bytes(S)) != hipSuccess)
        return 0;
    v = cus * per_cu;
    if (v > 0) __atomic_store_n(slot, v, __ATOMIC_RELAXED);
    return v;
}

// The same for the kernels that split the columns (S waves).
static int resident_split_workgroups(int shape, int S, int kind)
{
    static int cache[2][kKinds][kSplitMaxS + 1];
    int *slot = &cache[shape][kind][S];
    const void *fn = kSplitShapes[shape].fn[kind];
    int v = __atomic_load_n(slot, __ATOMIC_RELAXED);
    if (v > 0) return v;
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)stage_bytes(S)) != hipSuccess) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, S * 64, stage_bytes(S)) != hipSuccess) return 0;
    v = cus * per_cu;
    if (v > 0) __atomic_store_n(slot, v, __ATOMIC_RELAXED);
    return v;
}

int launch_mfma(const uint32_t *packed, const float *scales, const Layout &L, int bits_used, int frac_bits,
                int act_bits, const float *X0, int cols0, const float *X1, int cols1, const uint32_t *planes,
                int batch, float *Y, long long *A, bool pairs_out, const Epilogue &ep, hipStream_t st)
{
    MfmaArgs a;
    MfmaHead h;
    h.packed = packed; h.X0 = X0; a.X1 = X1; a.planes = planes; a.scales = scales; a.Y = Y; a.A = A;
    a.pairs_out = (A && pairs_out) ? 1 : 0;
    a.bias = ep.bias; a.relu = ep.relu; a.c_prev = ep.c_prev; a.h_out = ep.h_out; a.c_out = ep.c_out;
    a.gate_h = L.gate_h;
    // (the epilogue addresses the bias and the cell state with 32-bit byte offsets)
    if (ep.bias && L.rows >= (1 << 29)) return (int)hipErrorInvalidValue;
    if (ep.c_prev && (size_t)batch * (size_t)L.gate_h >= ((size_t)1 << 29)) return (int)hipErrorInvalidValue;
    h.packed_bytes = (uint32_t)packed_bytes(L);   // (the host API refuses matrices of 4 GiB and more)
    h.flags = (planes ? kPlanesGiven : 0u) | (X1 ? kSecondPart : 0u);
    h.layer_step = (uint32_t)(tile16_layer_stride(L) * 4);
    h.round_step = (uint32_t)(tile16_rowtile_stride(L) * 4);
    h.cols0 = cols0; a.cols1 = cols1;
    a.R = L.rows; h.rt_count = L.rt_count; h.cq = L.cq; a.cwp = L.cwp;
    h.m = bits_used;
    h.batch = batch;
    a.fscale = ldexpf(1.0f, frac_bits);
    a.imax = (act_bits == 32) ? INT32_MAX : (int32_t)((1u << (act_bits - 1)) - 1u);
    a.imin = -a.imax - 1;
    a.out_scale = ldexp(1.0, -frac_bits);
    // Vectors per operand: with at most 16 (8) activation bits two (four) vectors share an operand, if the call has
    // that many (planes that are given in memory are taken one vector per operand).
    int pk = planes ? 1 : (act_bits <= 8 ? 4 : (act_bits <= 16 ? 2 : 1));
    while (pk > 1 && pk / 2 >= batch) pk /= 2;
    const int slots = (batch + pk - 1) / pk;   // operands that the call fills
    // Bitlayer pairs when several vectors share the expanded weights (and for the parity hook of the pairs); the
    // kernels with packed operands are pair kernels (they multiply bitlayer by bitlayer when the per-layer sums are
    // asked for or the scales do not halve)
    bool pair = a.pairs_out || (!A && batch >= 2) || pk > 1;
    if (tuning().pair >= 0 && pk == 1) pair = a.pairs_out || (!A && tuning().pair != 0);
    if (is_pairs(L.layout)) pair = true;   // (the digit layout is read by the pair kernels, whatever the call)
    if (L.cols > kMaxColsPairs) return (int)hipErrorInvalidValue;   // (cannot happen: pairs cover every width)
    const int kind = !pair ? kSingle
                           : (pk == 1 ? kPairs : (pk == 2 ? kPairs2 : kPairs4)) + (is_pairs(L.layout) ? kDigits : 0);
    void *args[] = {&h.packed, &h.X0, &h.packed_bytes, &h.flags, &h.cols0, &h.batch, &h.layer_step, &h.round_step,
                    &h.rounds_per_wg, &h.rt_count, &h.cq, &h.m, &a};
    // Batches on wide rows take the columns in several passes (see SplitShape).
    // Beyond 8192 columns a wave has registers for the digit rows of two operands only (one beyond 16384 columns):
    // passes of four operands from five operands on (three beyond 16384 columns), of eight operands from seventeen on,
    // or earlier if that fills the workgroup with more waves (12288 columns: six waves with passes of 8192 columns,
    // eight with passes of 4096).  Up to 8192 columns the bit layout gains from eight operands per expanded word from
    // 33 operands on; the digit layout, whose expansion is cheaper, does not.
    // (Measured, bits_used 8, us per call.  Plain / passes of four: 16384 columns: batch 4 63 / 61, batch 8 113 / 98,
    // batch 64 807 / 645; 32768: batch 4 594 / 223, batch 64 7400 / 2400.  Passes of four / of eight, bit layout |
    // digit layout: 16384: batch 12 137 / 145 | 125 / 135, batch 24 270 / 225 | 240 / 209, batch 64 586 / 504 |
    // 502 / 475; 12288: batch 8 66 / 57 | 58 / 54, batch 64 398 / 289 | 342 / 263.  Plain / passes of eight at 8192:
    // batch 24 65 / 68, batch 32 79 / 77, batch 48 123 / 113, batch 64 156 / 136, batch 1024 2104 / 1873 | digit
    // layout: batch 32 68 / 72, batch 64 130 / 128, batch 1024 1778 / 1749.)
    int shape = -1;
    {
        const bool has4 = kSplitShapes[0].fn[kind] != nullptr, has8 = kSplitShapes[1].fn[kind] != nullptr;
        // (groups of eight must not leave many more operand places empty than groups of four would: 33 operands are
        // five groups of eight or nine of four, and 16-bit activations at batch 66, 33 operands, took 110 us in
        // groups of eight against 96 us)
        const bool fills8 = 8 * ((slots + 7) / 8) * 100 <= 4 * ((slots + 3) / 4) * 108;
        if (L.cq > kSplitChunks4) {
            const int waves4 = (split_chunks_per_part(L.cq, kSplitChunks4) + 1) / 2;
            const int waves8 = split_chunks_per_part(L.cq, kSplitChunks8);
            if (has8 && ((slots >= 17 && fills8) || (slots >= 5 && waves8 > waves4))) shape = 1;
            else if (has4 && (slots >= 5 || (L.cq > 2 * kSplitChunks4 && slots >= 3))) shape = 0;
        } else if (L.cq > kSplitChunks8 && has8 && !is_pairs(L.layout) && slots >= 33 && fills8) {
            shape = 1;
        }
    }
    if (tuning().split >= 0) {
        shape = -1;
        if (tuning().split == 4 && kSplitShapes[0].fn[kind] && slots >= 3) shape = 0;
        if (tuning().split == 8 && kSplitShapes[1].fn[kind] && slots >= 5) shape = 1;
    }
    if (shape >= 0) {
        const SplitShape &sh = kSplitShapes[shape];
        const int S = (split_chunks_per_part(L.cq, sh.chunks) + sh.nq - 1) / sh.nq;
        const int groups = (slots + sh.nv - 1) / sh.nv;
        int capacity = resident_split_workgroups(shape, S, kind);
        if (capacity < 1) return (int)hipErrorInvalidValue;
        if (tuning().wgs > 0) capacity = tuning().wgs;
        int wgs = capacity / groups;
        if (wgs < 1) wgs = 1;
        if (wgs > L.rt_count) wgs = L.rt_count;
        h.rounds_per_wg = (L.rt_count + wgs - 1) / wgs;
        wgs = (L.rt_count + h.rounds_per_wg - 1) / h.rounds_per_wg;
        const hipError_t e = hipLaunchKernel(sh.fn[kind], dim3((unsigned)wgs, (unsigned)groups), dim3((unsigned)S * 64),
                                             args, planes ? 0 : stage_bytes(S), st);
        return (int)(e != hipSuccess ? e : hipGetLastError());
    }
    int vi = pick_variant(L, slots, kind);
    if (vi < 0) return (int)hipErrorInvalidValue;
    const Variant &var = kVariants[vi];   // (the ring depth does not change a variant's occupancy: same registers +- a few)
    const int S = (L.cq + var.nq - 1) / var.nq;
    const int groups = (slots + var.nv - 1) / var.nv;
    // Workgroups: as many as are resident at once (so that every wave builds its planes once and the weight
    // stream never waits for a second round of workgroups to start), each with whole row tiles.
    int capacity = resident_workgroups(pick_ring(vi, 1 << 30, kind), S, kind);   // of the sibling that needs the most registers
    if (capacity < 1) return (int)hipErrorInvalidValue;
    if (tuning().wgs > 0) capacity = tuning().wgs;
    int wgs = capacity / groups;
    if (wgs < 1) wgs = 1;
    if (wgs > L.rt_count) wgs = L.rt_count;
    h.rounds_per_wg = (L.rt_count + wgs - 1) / wgs;
    wgs = (L.rt_count + h.rounds_per_wg - 1) / h.rounds_per_wg;
    const Variant &run = kVariants[pick_ring(vi, h.rounds_per_wg * (pair ? (bits_used + 1) / 2 : bits_used), kind)];
    const hipError_t e = hipLaunchKernel(run.fn[kind], dim3((unsigned)wgs, (unsigned)groups), dim3((unsigned)S * 64),
                                         args, planes ? 0 : stage_bytes(S), st);
    return (int)(e != hipSuccess ? e : hipGetLastError());
}

}  // namespace pb

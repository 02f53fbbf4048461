// The hot kernel on the matrix cores: the whole inference path of Algorithm 2 of the
// paper in one launch -- x_q = Int(x * 2^f), the bitwise transpose into bit planes
// (Section 3.4), the 1-bit products of Section 3.1 with the 32 planes of a vector
// batched as the second matrix operand ("one batched matrix product"), the plane
// weights [-2^31, 2^30 .. 2^0] and the scale-accumulation over the first `bits_used`
// bitlayers (the run-time knob of the abstract).
//
// Why the matrix cores: AND + popcount costs two vector-ALU lane operations per
// (32-bit weight word, plane); with 32 planes that is four times what the ALUs of
// this chip can do while HBM delivers the words.  The same 0/1 inner products are
// a dense contraction with N = 32 planes, and V_MFMA_SCALE_F32_16X16X128_F8F6F4 on
// FP4 (E2M1) operands does 32768 of them per instruction with exact results: the
// products are 0 or 1 and the fp32 accumulators count to 2^24.
//
// Operands.  A (16 x 128) = 16 planes x 128 columns, B (128 x 16) = 128 columns x
// 16 weight rows, D (16 x 16): lane l of D holds row j = l % 16 of the weights and
// the planes 4 * (l / 16) + v in its four registers v, so the plane weighting is
// arithmetic inside a lane.  Two instructions (planes 0-15 and 16-31) share one B.
// A lane's B operand is 32 columns of one weight row = ONE packed word, expanded
// from 1 bit to the 4-bit FP4 code per column with five ALU operations:
//     b0 = w & 0x11111111 (0.5)   b1 = w & 0x22222222 (1.0)
//     b2 = w & 0x44444444 (2.0)   b3 = (w >> 1) & 0x44444444 (2.0)
// and the plane operand carries the matching codes 2.0, 1.0, 0.5, 0.5 so that every
// product of two set bits is exactly 1.0.  Which column sits in which k slot does
// not matter as long as both operands agree.
//
// Mapping.  A wave owns a slice of the columns (NQ chunks of 512) for its whole life
// and keeps the expanded planes of that slice in registers; it streams the 1 KB
// blocks of its slice (see pb_layout.h) for row tile after row tile and bitlayer
// after bitlayer with 16-byte loads, several blocks in flight.  The waves of a
// workgroup are the slices of one row; their per-(row, bitlayer) sums meet in LDS
// through integer atomics, once per row tile, and one wave applies the layer scales
// and stores.  All integer results are exact, so they do not depend on the schedule.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "pb_kernels.h"

namespace pb {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct MfmaArgs {
    const uint32_t *packed;
    const float *X0, *X1;       // activations: row n is [X0[n][0..cols0) ; X1[n][0..cols1)]
    const uint32_t *planes;     // non-null: bit planes already in memory [batch][32][cwp] (prepared mode)
    const float *scales;
    float *Y;
    long long *A;
    const float *bias;          // [rows] or null: added to the fp32 result
    const float *c_prev;        // non-null: LSTM cell update instead of the store of Y (gate-interleaved rows)
    float *h_out, *c_out;
    int relu;                   // max(., 0) before the store of Y
    int gate_h;                 // gate-interleaved rows: H (packed row 16 t + 4 (u % 4) + gate = row gate * H + u), else 0
    size_t packed_bytes;
    uint32_t layer_step, round_step;   // bytes from one bitlayer of a row tile to the next, from one row tile to the next
    int cols0, cols1;
    int R, rt_count, cq, cwp;
    int m;                      // bitlayers to accumulate
    int batch;
    int rounds_per_wg;          // row tiles per workgroup
    float fscale;               // 2^frac_bits
    int imin, imax;             // range of the act_bits-bit fixed-point values
    double out_scale;           // 2^-frac_bits
};

// x_q = Int(x * 2^f) as a k-bit two's-complement value: toward zero, saturating, NaN -> 0.  V_CVT_I32_F32 does
// exactly that for k = 32 (out-of-range inputs saturate, NaN converts to 0); narrower k clamp the integer.
__device__ __forceinline__ int32_t to_fixed_point(float x, float fscale, int32_t imin, int32_t imax)
{
    int32_t r;
    const float p = x * fscale;   // exact: a power of two
    asm("v_cvt_i32_f32 %0, %1" : "=v"(r) : "v"(p));
    return min(max(r, imin), imax);
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_mov(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, CTRL, 0xf, 0xf, true);
}

// value of lane (l ^ J) for J < 16, inside each row of 16 lanes, on the vector ALU alone (DPP modifiers)
// value of lane L of the wave (a scalar)
template <int L>
__device__ __forceinline__ float lane_value(float v)
{
    return __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(v), L));
}

template <int J>
__device__ __forceinline__ uint32_t row_xor(uint32_t v)
{
    if constexpr (J == 8) return dpp_mov<0x128>(v);                     // row_ror:8
    else if constexpr (J == 4) return dpp_mov<0x1B>(dpp_mov<0x141>(v)); // row_half_mirror (l ^ 7), then quad_perm [3,2,1,0] (l ^ 3)
    else if constexpr (J == 2) return dpp_mov<0x4E>(v);                 // quad_perm [2,3,0,1]
    else return dpp_mov<0xB1>(v);                                       // quad_perm [1,0,3,2]
}

// sum over the 16 lanes of a row, in every lane (xor butterfly on the vector ALU)
__device__ __forceinline__ double row_sum16(double z)
{
#define PB_STEP(J)                                                                                  \
    {                                                                                               \
        const unsigned long long b = (unsigned long long)__double_as_longlong(z);                   \
        const uint32_t lo = row_xor<J>((uint32_t)b), hi = row_xor<J>((uint32_t)(b >> 32));          \
        z += __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));                \
    }
    PB_STEP(8) PB_STEP(4) PB_STEP(2) PB_STEP(1)
#undef PB_STEP
    return z;
}

// Per-lane constants of the 16 x 16 bit-matrix transpose across a row of 16 lanes (both 16-bit halves of a
// register at once): in stage J lanes l and l ^ J exchange the bit positions that have bit J set (lower lane)
// / clear (upper lane); keep = the positions a lane keeps, rot = right-rotation that moves the partner's bits
// into the others (>> J for the upper lane, << J for the lower).
struct TransposeConsts {
    uint32_t keep8, keep4, keep2, keep1;
    uint32_t rot8, rot4, rot2, rot1;
};

__device__ __forceinline__ TransposeConsts transpose_consts(int lane)
{
    TransposeConsts c;
    c.keep8 = (lane & 8) ? 0xFF00FF00u : 0x00FF00FFu; c.rot8 = (lane & 8) ? 8 : 24;
    c.keep4 = (lane & 4) ? 0xF0F0F0F0u : 0x0F0F0F0Fu; c.rot4 = (lane & 4) ? 4 : 28;
    c.keep2 = (lane & 2) ? 0xCCCCCCCCu : 0x33333333u; c.rot2 = (lane & 2) ? 2 : 30;
    c.keep1 = (lane & 1) ? 0xAAAAAAAAu : 0x55555555u; c.rot1 = (lane & 1) ? 1 : 31;
    return c;
}

template <int J>
__device__ __forceinline__ uint32_t transpose_stage(uint32_t x, uint32_t keep, uint32_t rot)
{
    const uint32_t other = row_xor<J>(x);
    const uint32_t moved = __builtin_amdgcn_alignbit(other, other, rot);
    return (x & keep) | (moved & ~keep);
}

// Lane r of a row holds, in each 16-bit half, 16 bits of one column; returns, in lane r, bit r of the 16 columns
// of the row (for each half).
__device__ __forceinline__ uint32_t bit_transpose16(uint32_t x, const TransposeConsts &c)
{
    x = transpose_stage<8>(x, c.keep8, c.rot8);
    x = transpose_stage<4>(x, c.keep4, c.rot4);
    x = transpose_stage<2>(x, c.keep2, c.rot2);
    x = transpose_stage<1>(x, c.keep1, c.rot1);
    return x;
}

// Plane word -> the four A-operand registers (FP4 codes 2.0, 1.0, 0.5, 0.5 facing the weight codes 0.5, 1.0, 2.0, 2.0)
__device__ __forceinline__ void expand_plane(uint32_t pw, u32x4 &dst)
{
    dst.x = (pw & 0x11111111u) << 2;
    dst.y = pw & 0x22222222u;
    dst.z = (pw & 0x44444444u) >> 2;
    dst.w = (pw >> 3) & 0x11111111u;
}

__device__ __forceinline__ v8i as_operand(const u32x4 v)
{
    v8i r = {(int)v.x, (int)v.y, (int)v.z, (int)v.w, 0, 0, 0, 0};   // FP4 operands use the first four registers
    return r;
}

__device__ __forceinline__ v8i weight_operand(uint32_t w)
{
    v8i r = {(int)(w & 0x11111111u), (int)(w & 0x22222222u), (int)(w & 0x44444444u),
             (int)((w >> 1) & 0x44444444u), 0, 0, 0, 0};
    return r;
}

__device__ __forceinline__ v4f mfma_fp4(const v8i a, const v8i b, const v4f c)
{
    // cbsz = blgp = 4: both operands FP4 (E2M1); block scales 2^0 (E8M0 code 127)
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 4, 4, 0, 0x7F, 0, 0x7F);
}

// NQ: chunks of 512 columns per wave; NV: activation vectors whose planes a wave keeps (each weight block is
// expanded once and multiplied with all of them); MAXS: most waves (column slices) per workgroup, which bounds
// the registers a wave may use; RU: units (row tile, bitlayer) whose blocks a wave has in flight.  The host picks
// RU <= the units a wave has, so that a short stream pays for no empty ring slots; 4 KB in flight per wave
// measured best (more requests in flight than that slow the short streams down and do not speed up the long ones).
// HI: planes 16-31 are computed.  Activations of at most 16 bits (Section 3.1: k = 8, 16) have planes 15-31 all
// equal to their sign plane, which together weigh -2^15: one matrix instruction per step instead of two, half the
// transpose, same integers.
template <int NQ, int NV, int MAXS, int RU, bool HI>
__global__ __launch_bounds__(MAXS * 64) void k_mfma(const MfmaArgs a)
{
    // Units requested before the activations have arrived (a head start that keeps HBM busy during the transpose);
    // the rest of the ring follows once the planes are built.
#ifndef PB_MFMA_PRE
#define PB_MFMA_PRE 2
#endif
    constexpr int PRE = NQ >= 4 ? (PB_MFMA_PRE < 1 ? PB_MFMA_PRE : 1) : (RU < PB_MFMA_PRE ? RU : PB_MFMA_PRE);
    // (low 16 planes, high 16 planes) sums per vector, bitlayer and row; two buffers, used by alternate row tiles
    __shared__ int2 abuf[2][NV][PB_MAX_BITS][kTileRows];
    __shared__ float s_scales[PB_MAX_BITS];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nwaves = blockDim.x >> 6;
    const int n0 = blockIdx.y * NV;                             // first activation vector of this workgroup
    const int m = a.m;
    const int q0 = wave * NQ;                                   // first chunk of this wave's column slice
    const int nq = min(NQ, a.cq - q0);                          // chunks it really has (>= 1 by construction)
    const int rt0 = blockIdx.x * a.rounds_per_wg;
    const int rounds = min(a.rounds_per_wg, a.rt_count - rt0);  // >= 1 by construction
    const int U = rounds * m;

    // layer scales, lane i holds scales[i]: the oldest load of the wave, so that no later wait is held up by it;
    // parked in LDS once the planes are built (the barrier before the first final sum orders that store)
    const float scv = (a.scales && lane < m) ? a.scales[lane] : 0.0f;

    // ---- the weight stream of this wave: unit u = (round r, bitlayer i), NQ blocks of 1 KB each ----
    const size_t base_off = (size_t)rt0 * a.round_step + (size_t)q0 * 1024;
    const char *base = reinterpret_cast<const char *>(a.packed) + base_off;
    const uint32_t avail = (uint32_t)(a.packed_bytes - base_off);
    const int voff = lane * 16;
    u32x4 ring[RU][NQ];
    uint32_t ld_soff = 0;
    int ld_i = 0, ld_u = 0;
    auto issue = [&](u32x4 (&dst)[NQ]) {
        // past the last unit, and for chunks beyond the end of a ragged last slice, the descriptor has 0 records:
        // every lane is out of range, the load returns 0 and moves no data (no branch, so the compiler counts
        // the loads in flight exactly)
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<char *>(base), 0, (ld_u < U && q < nq) ? (int)avail : 0, 0x00020000);
            dst[q] = __builtin_amdgcn_raw_buffer_load_b128(rs, voff + q * 1024, (int)ld_soff, /*nt*/ 2);
        }
        __builtin_amdgcn_sched_barrier(0x7);
        ++ld_u;
        if (++ld_i == m) { ld_i = 0; ld_soff += a.round_step - (uint32_t)(m - 1) * a.layer_step; }
        else ld_soff += a.layer_step;
    };

    // LDS sums start at zero.  The barrier that orders this is taken after every wave has REQUESTED its activations
    // and before any wave requests weights: the memory pipeline of a CU returns data in request order, so an
    // activation load queued behind another wave's weight loads (HBM misses) would arrive a memory latency late.
    auto zero_sums_and_meet = [&]() {
        for (int i = threadIdx.x; i < 2 * NV * PB_MAX_BITS * kTileRows; i += blockDim.x)
            (&abuf[0][0][0][0])[i] = make_int2(0, 0);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- the planes of this wave's slice, expanded to A operands, kept in registers ----
    // lane l = 16 * kb + p: planes p (lo) and 16 + p (hi) of the words 16 * q + 4 * kb + t
    const int kb = lane >> 4;
    u32x4 pa_lo[NV][NQ][4], pa_hi[NV][NQ][4];
    if (a.planes) {
        uint4 plo[NV][NQ], phi[NV][NQ];
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int n = min(n0 + v, a.batch - 1);
            const bool live = n0 + v < a.batch;
            const uint32_t *pl =
                a.planes + ((size_t)n * 32 + (lane & 15)) * (size_t)a.cwp + (size_t)q0 * 16 + 4 * kb;
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                plo[v][q] = phi[v][q] = make_uint4(0, 0, 0, 0);
                if (q < nq && live) {
                    plo[v][q] = *reinterpret_cast<const uint4 *>(pl + q * 16);
                    phi[v][q] = *reinterpret_cast<const uint4 *>(pl + (size_t)16 * a.cwp + q * 16);
                }
            }
        }
        zero_sums_and_meet();
#pragma unroll
        for (int k = 0; k < PRE; ++k) issue(ring[k]);
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const uint4 lo = plo[v][q], hi = phi[v][q];
                expand_plane(lo.x, pa_lo[v][q][0]); expand_plane(lo.y, pa_lo[v][q][1]);
                expand_plane(lo.z, pa_lo[v][q][2]); expand_plane(lo.w, pa_lo[v][q][3]);
                if (HI) {
                    expand_plane(hi.x, pa_hi[v][q][0]); expand_plane(hi.y, pa_hi[v][q][1]);
                    expand_plane(hi.z, pa_hi[v][q][2]); expand_plane(hi.w, pa_hi[v][q][3]);
                }
            }
    } else {
        // Algorithm 2: x_q = Int(x * 2^f); then the bitwise transpose, 32 columns x 32 bits at a time in each
        // half of the wave: lane (half H, column c) converts column c of word 16 q + 4 (2 H + e) + t, e = 0, 1.
        // V_PERMLANE16_SWAP hands the even rows of 16 lanes both 16-column halves of the e = 0 word and the odd
        // rows those of the e = 1 word, which is the first stage of the 32 x 32 transpose; the other four stages
        // stay inside a row.  Lane (kb, p) ends with planes p and 16 + p of word 16 q + 4 kb + t.
        // Buffer loads return 0 beyond the end of a vector, and for the vectors beyond the end of the batch.
        const int colb = (32 * (16 * q0 + 8 * (lane >> 5)) + (lane & 31)) * 4;   // byte offset of (q = 0, e = 0, t = 0)
        uint32_t xv[NV][NQ][4][2];
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int n = min(n0 + v, a.batch - 1);
            const bool live = n0 + v < a.batch;
            const __amdgpu_buffer_rsrc_t rx0 = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<float *>(a.X0 + (size_t)n * a.cols0), 0, live ? a.cols0 * 4 : 0, 0x00020000);
#pragma unroll
            for (int q = 0; q < NQ; ++q)
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int e = 0; e < 2; ++e)
                        xv[v][q][t][e] =
                            __builtin_amdgcn_raw_buffer_load_b32(rx0, colb + 128 * (16 * q + 4 * e + t), 0, 0);
        }
        // Second part of a concatenated input [X0 ; X1]: at most one of the two loads of a column is in range.
        // Columns of the first part would have negative offsets here; those are clamped and the value dropped
        // (a negative register offset that an instruction offset brings back above zero is not range-checked
        // lane by lane on this hardware).
        uint32_t xw[NV][NQ][4][2];
        const int colb1 = colb - a.cols0 * 4;
        if (a.X1) {
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const int n = min(n0 + v, a.batch - 1);
                const bool live = n0 + v < a.batch;
                const __amdgpu_buffer_rsrc_t rx1 = __builtin_amdgcn_make_buffer_rsrc(
                    const_cast<float *>(a.X1 + (size_t)n * a.cols1), 0, live ? a.cols1 * 4 : 0, 0x00020000);
#pragma unroll
                for (int q = 0; q < NQ; ++q)
#pragma unroll
                    for (int t = 0; t < 4; ++t)
#pragma unroll
                        for (int e = 0; e < 2; ++e)
                            xw[v][q][t][e] = __builtin_amdgcn_raw_buffer_load_b32(
                                rx1, max(colb1 + 128 * (16 * q + 4 * e + t), 0), 0, 0);
            }
        }
        zero_sums_and_meet();
#pragma unroll
        for (int k = 0; k < PRE; ++k) issue(ring[k]);
        const TransposeConsts tc = transpose_consts(lane);
        if (a.X1) {
#pragma unroll
            for (int v = 0; v < NV; ++v)
#pragma unroll
                for (int q = 0; q < NQ; ++q)
#pragma unroll
                    for (int t = 0; t < 4; ++t)
#pragma unroll
                        for (int e = 0; e < 2; ++e)
                            xv[v][q][t][e] |= colb1 + 128 * (16 * q + 4 * e + t) >= 0 ? xw[v][q][t][e] : 0u;
        }
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int q = 0; q < NQ; ++q)
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const uint32_t X =
                        (uint32_t)to_fixed_point(__uint_as_float(xv[v][q][t][0]), a.fscale, a.imin, a.imax);
                    const uint32_t Y =
                        (uint32_t)to_fixed_point(__uint_as_float(xv[v][q][t][1]), a.fscale, a.imin, a.imax);
                    const auto sw = __builtin_amdgcn_permlane16_swap(X, Y, false, false);
                    // even rows: (columns 0-15, columns 16-31) of the e = 0 word; odd rows: of the e = 1 word
                    const uint32_t c_lo = sw[0], c_hi = sw[1];
                    const uint32_t lo = (c_lo & 0xFFFFu) | (c_hi << 16);         // bits 0-15 of the 32 columns
                    const uint32_t hi = (c_hi & 0xFFFF0000u) | (c_lo >> 16);     // bits 16-31
                    expand_plane(bit_transpose16(lo, tc), pa_lo[v][q][t]);
                    if (HI) expand_plane(bit_transpose16(hi, tc), pa_hi[v][q][t]);
                }
    }
    if (wave == 0 && lane < PB_MAX_BITS) s_scales[lane] = scv;
    __builtin_amdgcn_sched_barrier(0);   // the rest of the ring is requested after the activations have arrived
#pragma unroll
    for (int k = PRE; k < RU; ++k) issue(ring[k]);

    // per-lane plane weights: registers c of the low / high instruction hold planes 4 kb + c / 16 + 4 kb + c
    float kl[4], kh[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        kl[c] = (float)(1 << (4 * kb + c));
        kh[c] = (kb == 3 && c == 3) ? -kl[c] : kl[c];    // plane 31 weighs -2^31 (Algorithm 2)
    }
    if (!HI && kb == 3) kl[3] = -kl[3];                  // 16-bit activations: plane 15 stands for planes 15-31, -2^15

    const int j = lane & 15;
    int pi = 0, pr = 0;   // bitlayer and round of the unit being multiplied
    for (int u0 = 0; u0 < U; u0 += RU) {
#pragma unroll
        for (int k = 0; k < RU; ++k) {
            if (u0 + k < U) {
                v4f acc_lo[NV], acc_hi[NV];
#pragma unroll
                for (int v = 0; v < NV; ++v) acc_lo[v] = acc_hi[v] = v4f{0.f, 0.f, 0.f, 0.f};
                // (chunks beyond a ragged last slice multiply zero planes by zero weights)
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    const u32x4 w = ring[k][q];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const v8i b = weight_operand(w[t]);
#pragma unroll
                        for (int v = 0; v < NV; ++v) {
                            acc_lo[v] = mfma_fp4(as_operand(pa_lo[v][q][t]), b, acc_lo[v]);
                            if (HI) acc_hi[v] = mfma_fp4(as_operand(pa_hi[v][q][t]), b, acc_hi[v]);
                        }
                    }
                }
                // plane weighting inside the lane.  Counts are <= 2048 (a slice has at most 2048 columns), so
                // c0 + 2 c1 + 4 c2 +- 8 c3 < 2^15 and its multiple by 2^(4 kb) is exact in fp32 and < 2^27.
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    const float lo_f = acc_lo[v][0] * kl[0] + acc_lo[v][1] * kl[1] + acc_lo[v][2] * kl[2] +
                                       acc_lo[v][3] * kl[3];
                    const float hi_f = acc_hi[v][0] * kh[0] + acc_hi[v][1] * kh[1] + acc_hi[v][2] * kh[2] +
                                       acc_hi[v][3] * kh[3];
                    int2 *dst = &abuf[pr & 1][v][pi][j];
                    atomicAdd(&dst->x, (int)lo_f);
                    if (HI) atomicAdd(&dst->y, (int)hi_f);
                }
                if (++pi == m) {
                    // The row tile is complete in every slice: scale and store it.  (The barrier per row tile also
                    // keeps the waves of a workgroup on one contiguous region of the weight stream; letting them
                    // drift apart over several row tiles measured 5-15 % slower.)
                    // A task = (vector, four rows); lane = (row of the four, bitlayer): every lane converts one
                    // (row, bitlayer) sum, the 16 lanes of a row add up their scaled terms.  The waves share the
                    // 4 * NV tasks out, so that none of them is late for the next barrier.
                    pi = 0;
                    __syncthreads();
                    const int rq = lane >> 4, il = lane & 15;
                    for (int task = wave; task < 4 * NV; task += nwaves) {
                        const int v = task >> 2, jrow = (task & 3) * 4 + rq, n = n0 + v;
                        const int prow = (rt0 + pr) * kTileRows + jrow;
                        const int row = a.gate_h ? gates_matrix_row(prow, a.gate_h) : prow;
                        const bool live = n < a.batch && row >= 0 && row < a.R;
                        int2 s = make_int2(0, 0);
                        if (il < m) {
                            int2 *src = &abuf[pr & 1][v][il][jrow];
                            s = *src;
                            *src = make_int2(0, 0);
                        }
                        // A_i = lo + hi * 2^16 exactly: 0 <= lo < 2^31 (unsigned), |hi| <= 2^30; with 16 planes lo
                        // carries the sign plane itself, |lo| < 2^30, and hi is 0
                        const long long lo = HI ? (long long)(uint32_t)s.x : (long long)s.x;
                        if (a.A) {
                            if (live && il < m)
                                a.A[((size_t)il * a.batch + n) * (size_t)a.R + row] = lo + ((long long)s.y << 16);
                            continue;
                        }
                        const double z = row_sum16((double)s_scales[il] * ((double)lo + (double)s.y * 65536.0));
                        float y = (float)(z * a.out_scale);
                        if (a.bias && live) y += a.bias[row];
                        if (a.c_prev) {
                            // LSTM cell: the four rows of the task are the gates i, f, g, o of one unit (row = unit
                            // for gate i); lane 0 updates the unit
                            const float gi = lane_value<0>(y), gf = lane_value<16>(y);
                            const float gg = lane_value<32>(y), go = lane_value<48>(y);
                            if (lane == 0 && live) {
                                const size_t at = (size_t)n * a.gate_h + (size_t)row;
                                const float cn = sigmoid_f(gf) * a.c_prev[at] + sigmoid_f(gi) * tanhf(gg);
                                a.c_out[at] = cn;
                                a.h_out[at] = sigmoid_f(go) * tanhf(cn);
                            }
                        } else {
                            if (a.relu) y = fmaxf(y, 0.0f);
                            if (live && il == 0) a.Y[(size_t)n * a.R + row] = y;
                        }
                    }
                    ++pr;
                }
            }
            issue(ring[k]);
        }
    }
}

// The kernel variants: (chunks per wave, vectors per wave, most slices per workgroup, ring depth in units).
struct Variant {
    int nq, nv, maxs, ru;
    const void *fn, *fn16;    // 32 planes, 16 planes
};
#define PB_VARIANT(NQ, NV, MAXS, RU)                                                          \
    {NQ, NV, MAXS, RU, reinterpret_cast<const void *>(k_mfma<NQ, NV, MAXS, RU, true>),        \
     reinterpret_cast<const void *>(k_mfma<NQ, NV, MAXS, RU, false>)}
static const Variant kVariants[] = {
    PB_VARIANT(1, 1, 16, 1), PB_VARIANT(1, 1, 16, 2), PB_VARIANT(1, 1, 16, 4),
    PB_VARIANT(1, 2, 8, 1),  PB_VARIANT(1, 2, 8, 2),  PB_VARIANT(1, 2, 8, 4),
    PB_VARIANT(1, 4, 8, 1),  PB_VARIANT(1, 4, 8, 2),  PB_VARIANT(1, 4, 8, 4),
    PB_VARIANT(2, 1, 16, 1), PB_VARIANT(2, 1, 16, 2),
    PB_VARIANT(2, 2, 8, 1),  PB_VARIANT(2, 2, 8, 2),
    PB_VARIANT(4, 1, 8, 1),  PB_VARIANT(4, 1, 8, 2),
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

// As many vectors per wave as the batch has and the registers allow (each weight block is then read and expanded
// once for all of them), then the smallest slice (most waves per row, shortest transpose per wave) whose slice
// count fits a workgroup; ring depth 1 (the deeper rings are picked once the units per wave are known).
static int pick_variant(const Layout &L, int batch)
{
    int want_nq = 0, want_nv = 0;
    if (const char *e = getenv("PB_TUNE_NQ")) want_nq = atoi(e);
    if (const char *e = getenv("PB_TUNE_NV")) want_nv = atoi(e);
    int best = -1;
    for (int i = 0; i < kNumVariants; ++i) {
        const Variant &v = kVariants[i];
        if (v.ru != 1) continue;
        if ((L.cq + v.nq - 1) / v.nq > v.maxs) continue;
        if (want_nq && v.nq != want_nq) continue;
        if (want_nv ? v.nv != want_nv : (v.nv > 1 && v.nv / 2 >= batch)) continue;   // no more than one empty half
        if (best < 0 || v.nv > kVariants[best].nv || (v.nv == kVariants[best].nv && v.nq < kVariants[best].nq))
            best = i;
    }
    return best;
}

// The sibling of variant `vi` with the deepest ring that a wave with `units` units fills.
static int pick_ring(int vi, int units)
{
    int want = 0;
    if (const char *e = getenv("PB_TUNE_RU")) want = atoi(e);
    int best = vi;
    for (int i = 0; i < kNumVariants; ++i) {
        const Variant &v = kVariants[i];
        if (v.nq != kVariants[vi].nq || v.nv != kVariants[vi].nv) continue;
        if (want ? v.ru == want : (v.ru <= units && v.ru > kVariants[best].ru)) best = i;
    }
    return best;
}

// Workgroups of S waves that fit on the device at once (occupancy does not change while the process lives, so it
// is looked up once per kernel variant and workgroup size).
static int resident_workgroups(int variant, int S)
{
    static int cache[kNumVariants][kMaxSlices + 1];
    int v = __atomic_load_n(&cache[variant][S], __ATOMIC_RELAXED);
    if (v > 0) return v;
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kVariants[variant].fn, S * 64, 0) != hipSuccess)
        return 0;
    v = cus * per_cu;
    if (v > 0) __atomic_store_n(&cache[variant][S], v, __ATOMIC_RELAXED);
    return v;
}

int launch_mfma(const uint32_t *packed, const float *scales, const Layout &L, int bits_used, int frac_bits,
                int act_bits, const float *X0, int cols0, const float *X1, int cols1, const uint32_t *planes,
                int batch, float *Y, long long *A, const Epilogue &ep, hipStream_t st)
{
    MfmaArgs a;
    a.packed = packed; a.X0 = X0; a.X1 = X1; a.planes = planes; a.scales = scales; a.Y = Y; a.A = A;
    a.bias = ep.bias; a.relu = ep.relu; a.c_prev = ep.c_prev; a.h_out = ep.h_out; a.c_out = ep.c_out;
    a.gate_h = L.gate_h;
    a.packed_bytes = packed_bytes(L);
    a.layer_step = (uint32_t)(tile16_layer_stride(L) * 4);
    a.round_step = (uint32_t)(tile16_rowtile_stride(L) * 4);
    a.cols0 = cols0; a.cols1 = cols1;
    a.R = L.rows; a.rt_count = L.rt_count; a.cq = L.cq; a.cwp = L.cwp;
    a.m = bits_used;
    a.batch = batch;
    a.fscale = ldexpf(1.0f, frac_bits);
    a.imax = (act_bits == 32) ? INT32_MAX : (int32_t)((1u << (act_bits - 1)) - 1u);
    a.imin = -a.imax - 1;
    a.out_scale = ldexp(1.0, -frac_bits);
    int vi = pick_variant(L, batch);
    if (vi < 0) return (int)hipErrorInvalidValue;
    const Variant &var = kVariants[vi];   // (the ring depth does not change a variant's occupancy: same registers +- a few)
    const int S = (L.cq + var.nq - 1) / var.nq;
    const int groups = (batch + var.nv - 1) / var.nv;
    // Workgroups: as many as are resident at once (so that every wave builds its planes once and the weight
    // stream never waits for a second round of workgroups to start), each with whole row tiles.
    int capacity = resident_workgroups(pick_ring(vi, 1 << 30), S);   // of the sibling that needs the most registers
    if (capacity < 1) return (int)hipErrorInvalidValue;
    if (const char *e = getenv("PB_TUNE_WGS")) capacity = atoi(e);
    int wgs = capacity / groups;
    if (wgs < 1) wgs = 1;
    if (wgs > L.rt_count) wgs = L.rt_count;
    a.rounds_per_wg = (L.rt_count + wgs - 1) / wgs;
    wgs = (L.rt_count + a.rounds_per_wg - 1) / a.rounds_per_wg;
    void *args[] = {&a};
    const Variant &run = kVariants[pick_ring(vi, a.rounds_per_wg * bits_used)];
    const hipError_t e = hipLaunchKernel(act_bits > 16 ? run.fn : run.fn16, dim3((unsigned)wgs, (unsigned)groups), dim3((unsigned)S * 64), args,
                                         0, st);
    return (int)(e != hipSuccess ? e : hipGetLastError());
}

}  // namespace pb

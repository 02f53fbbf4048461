// Offline preprocessing kernels (Algorithm 1 of the paper): quantize-round the
// fp32 weights to B-bit two's-complement codes (Section 3.3), split the codes
// into B bitlayers, sign layer first (Section 3.2), and pack 32 columns per word
// (Section 3.4).  Not on the timed path ("done offline", Section 3.3).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pb_kernels.h"

namespace pb {

// Scratch for the reductions of the quantizers: 64 uint64 at the start of `packed` (every packed matrix is at
// least 512 bytes; the packing kernel overwrites them last).
enum { kSlotAbsMax = 0, kSlotMax = 1, kSlotMin = 2, kSlotAbsSum = 3, kSlotClip = 4, kScratchWords = 64 };
constexpr int kClipSteps = 32;

__global__ void k_fill_u64(unsigned long long *p, int n, unsigned long long v)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = (i == kSlotMin) ? ~0ull : v;
}

// a float as an unsigned key that orders like the float (NaN excluded by the caller)
__device__ __forceinline__ uint32_t ordered_key(float f)
{
    const uint32_t b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float from_ordered_key(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

// max |W|, max W and min W in one pass (Section 3.3: the step of every quantizer comes from these).
// 16-byte loads, one set of atomics per workgroup.
__global__ __launch_bounds__(256) void k_stats(const float *__restrict__ W, size_t n, unsigned long long *scratch)
{
    __shared__ uint32_t part[3][4];
    uint32_t am = 0, hi = 0, lo = 0xFFFFFFFFu;
    auto take = [&](float w) {
        if (w == w) {
            const uint32_t a = __float_as_uint(fabsf(w)), k = ordered_key(w);
            am = a > am ? a : am;
            hi = k > hi ? k : hi;
            lo = k < lo ? k : lo;
        }
    };
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const size_t n4 = n / 4;
    const float4 *W4 = reinterpret_cast<const float4 *>(W);   // W is 16-byte aligned (checked on the host)
    for (size_t i = tid; i < n4; i += stride) {
        const float4 w = W4[i];
        take(w.x); take(w.y); take(w.z); take(w.w);
    }
    for (size_t i = n4 * 4 + tid; i < n; i += stride) take(W[i]);
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t a = (uint32_t)__shfl_xor((int)am, off, 64), h = (uint32_t)__shfl_xor((int)hi, off, 64);
        const uint32_t l = (uint32_t)__shfl_xor((int)lo, off, 64);
        am = a > am ? a : am;
        hi = h > hi ? h : hi;
        lo = l < lo ? l : lo;
    }
    if ((threadIdx.x & 63) == 0) {
        part[0][threadIdx.x >> 6] = am; part[1][threadIdx.x >> 6] = hi; part[2][threadIdx.x >> 6] = lo;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w) {
            am = part[0][w] > am ? part[0][w] : am;
            hi = part[1][w] > hi ? part[1][w] : hi;
            lo = part[2][w] < lo ? part[2][w] : lo;
        }
        atomicMax(&scratch[kSlotAbsMax], (unsigned long long)am);
        atomicMax(&scratch[kSlotMax], (unsigned long long)hi);
        atomicMin(&scratch[kSlotMin], (unsigned long long)lo);
    }
}

__device__ __forceinline__ int quantize_code(float w, float d, int qmin, int qmax)
{
    float r = rintf(w / d);  // IEEE divide, round half to even
    if (r != r) return 0;
    if (r >= (float)qmax) return qmax;
    if (r <= (float)qmin) return qmin;
    return (int)r;
}

// trunc(|a| * 2^(30 - e)) for |a| < 2^(e + 1): an integer below 2^31, so that the sums below are exact in 64 bits
// and do not depend on the order of the additions
__device__ __forceinline__ unsigned long long fix30(float a, int e)
{
    const float t = truncf(ldexpf(fabsf(a), 30 - e));
    return (t != t) ? 0ull : (unsigned long long)t;
}

__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v)
{
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)v, off, 64);
        const uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)(v >> 32), off, 64);
        v += ((unsigned long long)hi << 32) | lo;
    }
    return v;
}

// 1-bit +-1 code (Section 3.3): sum of |W| for the scale d = mean |W|
__global__ __launch_bounds__(256) void k_abs_sum(const float *__restrict__ W, size_t n, unsigned long long *scratch)
{
    const float M = __uint_as_float((uint32_t)scratch[kSlotAbsMax]);
    const int e = M > 0.0f ? ilogbf(M) : 0;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    unsigned long long s = 0;
    for (; i < n; i += stride) {
        const float w = W[i];
        if (w == w) s += fix30(w, e);
    }
    s = wave_sum_u64(s);
    if ((threadIdx.x & 63) == 0 && s) atomicAdd(&scratch[kSlotAbsSum], s);
}

// clipping search (Section 3.3): summed |W - d_k q| for the thresholds T_k = max|W| k / 32, k = 1..32
__global__ __launch_bounds__(256) void k_clip_err(const float *__restrict__ W, size_t n, int bits,
                                                  unsigned long long *scratch)
{
    const float M = __uint_as_float((uint32_t)scratch[kSlotAbsMax]);
    if (M == 0.0f) return;
    const int e = ilogbf(M);
    const int qmax = (1 << (bits - 1)) - 1, qmin = -(1 << (bits - 1));
    const float qm = (float)(qmax > 0 ? qmax : 1);
    unsigned long long acc[kClipSteps];
#pragma unroll
    for (int k = 0; k < kClipSteps; ++k) acc[k] = 0;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) {
        const float w = W[i];
        if (w != w) continue;
#pragma unroll
        for (int k = 0; k < kClipSteps; ++k) {
            const float d = __fdiv_rn(__fmul_rn(M, __fmul_rn((float)(k + 1), 0.03125f)), qm);
            const float p = __fmul_rn(d, (float)quantize_code(w, d, qmin, qmax));
            acc[k] += fix30(__fsub_rn(w, p), e);
        }
    }
#pragma unroll
    for (int k = 0; k < kClipSteps; ++k) {
        const unsigned long long s = wave_sum_u64(acc[k]);
        if ((threadIdx.x & 63) == 0 && s) atomicAdd(&scratch[kSlotClip + k], s);
    }
}

// the step d of the chosen quantizer, left in scales[0] for the packing kernel
__global__ void k_step(const unsigned long long *scratch, int bits, int quantizer, size_t n, float *scales)
{
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    const float M = __uint_as_float((uint32_t)scratch[kSlotAbsMax]);
    const int qmax = (1 << (bits - 1)) - 1;
    const float qm = (float)(qmax > 0 ? qmax : 1);
    float d;
    if (quantizer == PB_QUANT_RANGE) {
        const float hi = from_ordered_key((uint32_t)scratch[kSlotMax]), lo = from_ordered_key((uint32_t)scratch[kSlotMin]);
        d = (scratch[kSlotMax] != 0 && hi > lo) ? __fdiv_rn(__fsub_rn(hi, lo), (float)(1 << (bits - 1))) : 1.0f;
    } else if (quantizer == PB_QUANT_SIGN) {
        const int e = M > 0.0f ? ilogbf(M) : 0;
        d = (float)(ldexp((double)scratch[kSlotAbsSum], e - 30) / (double)n);
    } else if (quantizer == PB_QUANT_CLIP_SEARCH && M != 0.0f) {
        int best = kClipSteps;
        unsigned long long best_err = scratch[kSlotClip + kClipSteps - 1];
        for (int k = kClipSteps - 1; k >= 1; --k)
            if (scratch[kSlotClip + k - 1] < best_err) { best = k; best_err = scratch[kSlotClip + k - 1]; }
        d = __fdiv_rn(__fmul_rn(M, __fmul_rn((float)best, 0.03125f)), qm);
    } else {
        d = (M == 0.0f) ? 1.0f : __fdiv_rn(M, qm);
    }
    scales[0] = d;
}

// One wave per (packed row, 64 columns): a lane quantizes one weight (a coalesced 256-byte read), the ballot of
// bit B-1-i over the wave IS two packed words of bitlayer i; lane i keeps and stores them (8 bytes).
__global__ __launch_bounds__(256) void k_pack(const float *__restrict__ W, uint32_t layout, int rows, int cols,
                                              int bits, int cwp, int rows_p, int gate_h, size_t layer_words,
                                              int quantizer, const float *__restrict__ step,
                                              uint32_t *__restrict__ packed)
{
    const int lane = threadIdx.x & 63;
    const int groups = cwp / 2;
    const long long tasks = (long long)rows_p * groups;
    const long long wave0 = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const long long nwaves = ((long long)gridDim.x * blockDim.x) >> 6;
    const float d = *step;
    const int qmax = (1 << (bits - 1)) - 1, qmin = -(1 << (bits - 1));
    for (long long task = wave0; task < tasks; task += nwaves) {
        const int pr = (int)(task / groups), g = (int)(task % groups);
        const int r = gate_h ? gates_matrix_row(pr, gate_h) : pr;   // matrix row (-1 or >= rows: padding)
        const int c = 64 * g + lane;
        uint32_t u = 0;
        if (r >= 0 && r < rows && c < cols) {
            const float w = W[(size_t)r * (size_t)cols + c];
            u = (uint32_t)(quantizer == PB_QUANT_SIGN ? ((w >= 0.0f || w != w) ? 1 : -1) : quantize_code(w, d, qmin, qmax));
        }
        uint32_t lo = 0, hi = 0;
        for (int i = 0; i < bits; ++i) {
            const unsigned long long bal = __ballot((u >> (bits - 1 - i)) & 1u);
            lo = (lane == i) ? (uint32_t)bal : lo;
            hi = (lane == i) ? (uint32_t)(bal >> 32) : hi;
        }
        int stored = bits;
        if (is_pairs(layout)) {
            // lanes 2p, 2p + 1 hold the bitlayers of pair p (zeros beyond the last bitlayer); the even lane ends up
            // with the digits of the even columns, the odd lane with those of the odd columns, for both words
            stored = (bits + 1) & ~1;
            if (lane == 0) { lo = ~lo; hi = ~hi; }      // the sign bitlayer enters as 1 - w
            const uint32_t plo = (uint32_t)__shfl_xor((int)lo, 1, 64), phi = (uint32_t)__shfl_xor((int)hi, 1, 64);
            const bool upper = !(lane & 1);              // this lane holds the upper bitlayer of its pair
            uint32_t e0, o0, e1, o1;
            digits_of_pair(upper ? lo : plo, upper ? plo : lo, &e0, &o0);   // columns 0-31 of the group
            digits_of_pair(upper ? hi : phi, upper ? phi : hi, &e1, &o1);   // columns 32-63
            lo = upper ? e0 : o0;
            hi = upper ? e1 : o1;
        }
        if (lane < stored)
            *reinterpret_cast<uint2 *>(packed + word_index(layout, cwp, layer_words, lane, pr, 2 * g)) = make_uint2(lo, hi);
    }
}

// reads the step from scales[0] (where k_step left it) and writes the layer scales
__global__ void k_scales(float *scales, int bits)
{
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    const float d = scales[0];
    for (int i = 0; i < bits; ++i) {
        float v = d * ldexpf(1.0f, bits - 1 - i);
        scales[i] = (i == 0) ? -v : v;
    }
}

__global__ __launch_bounds__(256) void k_unpack(const uint32_t *__restrict__ packed, uint32_t layout, int rows, int cols,
                                                int bits, int cwp, int gate_h, size_t layer_words,
                                                int32_t *__restrict__ q)
{
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)rows * (size_t)cols) return;
    int r = (int)(idx / (size_t)cols);
    int c = (int)(idx % (size_t)cols);
    uint32_t u = 0;
    const int pr = gate_h ? gates_packed_row(r, gate_h) : r;
    for (int i = 0; i < bits; ++i) {
        uint32_t word;
        if (is_pairs(layout)) {
            uint32_t upper, lower;
            pair_of_digits(packed[word_index(layout, cwp, layer_words, i & ~1, pr, c >> 5)],
                           packed[word_index(layout, cwp, layer_words, i | 1, pr, c >> 5)], &upper, &lower);
            word = (i & 1) ? lower : (i == 0 ? ~upper : upper);
        } else {
            word = packed[word_index(layout, cwp, layer_words, i, pr, c >> 5)];
        }
        u |= ((word >> (c & 31)) & 1u) << (bits - 1 - i);
    }
    int32_t v = (int32_t)(u << (32 - bits)) >> (32 - bits);  // sign-extend the B-bit code
    q[idx] = v;
}

int launch_quantize_pack(const float *W, const Layout &L, int quantizer, uint32_t *packed, float *scales,
                         hipStream_t st)
{
    const size_t n = (size_t)L.rows * (size_t)L.cols;
    unsigned long long *scratch = reinterpret_cast<unsigned long long *>(packed);
    hipLaunchKernelGGL(k_fill_u64, dim3(1), dim3(kScratchWords), 0, st, scratch, (int)kScratchWords, 0ull);
    int blocks = (int)((n + 256 * 16 - 1) / (256 * 16));
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(k_stats, dim3(blocks < 1024 ? blocks : 1024), dim3(256), 0, st, W, n, scratch);
    if (quantizer == PB_QUANT_SIGN) hipLaunchKernelGGL(k_abs_sum, dim3(blocks), dim3(256), 0, st, W, n, scratch);
    if (quantizer == PB_QUANT_CLIP_SEARCH)
        hipLaunchKernelGGL(k_clip_err, dim3(blocks), dim3(256), 0, st, W, n, L.bits, scratch);
    hipLaunchKernelGGL(k_step, dim3(1), dim3(64), 0, st, scratch, L.bits, quantizer, n, scales);
    const long long tasks = (long long)L.rows_p * (L.cwp / 2);
    long long pblocks = (tasks + 3) / 4;            // four waves per block, one task per wave and pass
    if (pblocks > 16384) pblocks = 16384;
    hipLaunchKernelGGL(k_pack, dim3((unsigned)pblocks), dim3(256), 0, st, W, L.layout, L.rows, L.cols, L.bits, L.cwp,
                       L.rows_p, L.gate_h, L.layer_words, quantizer, scales, packed);
    hipLaunchKernelGGL(k_scales, dim3(1), dim3(64), 0, st, scales, L.bits);
    return (int)hipGetLastError();
}

int launch_unpack(const uint32_t *packed, const Layout &L, int32_t *q, hipStream_t st)
{
    size_t n = (size_t)L.rows * (size_t)L.cols;
    hipLaunchKernelGGL(k_unpack, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, packed, L.layout, L.rows, L.cols,
                       L.bits, L.cwp, L.gate_h, L.layer_words, q);
    return (int)hipGetLastError();
}

}  // namespace pb

// Offline preprocessing kernels (Algorithm 1 of the paper): quantize-round the
// fp32 weights to B-bit two's-complement codes (Section 3.3), split the codes
// into B bitlayers, sign layer first (Section 3.2), and pack 32 columns per word
// (Section 3.4).  Not on the timed path ("done offline", Section 3.3).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pb_kernels.h"

namespace pb {

__global__ void k_fill_u32(uint32_t *p, size_t n, uint32_t v)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

// max |W| as the bit pattern of a non-negative float (orders like an unsigned integer)
__global__ __launch_bounds__(256) void k_absmax(const float *__restrict__ W, size_t n, uint32_t *slot)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    uint32_t m = 0;
    for (; i < n; i += stride) {
        float a = fabsf(W[i]);
        if (a == a) {
            uint32_t b = __float_as_uint(a);
            m = b > m ? b : m;
        }
    }
    for (int off = 32; off > 0; off >>= 1) {
        uint32_t o = (uint32_t)__shfl_xor((int)m, off, 64);
        m = o > m ? o : m;
    }
    if ((threadIdx.x & 63) == 0 && m != 0) atomicMax(slot, m);
}

__device__ __forceinline__ float grid_step(float M, int bits)
{
    int qmax = (1 << (bits - 1)) - 1;
    return (M == 0.0f) ? 1.0f : M / (float)(qmax > 0 ? qmax : 1);
}

__device__ __forceinline__ int quantize_code(float w, float d, int bits)
{
    int qmax = (1 << (bits - 1)) - 1;
    int qmin = -(1 << (bits - 1));
    float r = rintf(w / d);  // IEEE divide, round half to even
    if (r != r) return 0;
    if (r >= (float)qmax) return qmax;
    if (r <= (float)qmin) return qmin;
    return (int)r;
}

// one thread per (padded row, padded word): builds that word of every bitlayer
__global__ __launch_bounds__(256) void k_pack(const float *__restrict__ W, uint32_t layout, int rows, int cols,
                                              int bits, int cw, int cwp, int rows_p, int gate_h, size_t layer_words,
                                              const uint32_t *__restrict__ absmax_slot, uint32_t *__restrict__ packed)
{
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)rows_p * (size_t)cwp;
    if (idx >= total) return;
    const int pr = (int)(idx / (size_t)cwp);       // packed row
    int w = (int)(idx % (size_t)cwp);
    const int r = gate_h ? gates_matrix_row(pr, gate_h) : pr;   // matrix row (-1 or >= rows: padding)
    uint32_t wd[PB_MAX_BITS];
#pragma unroll
    for (int i = 0; i < PB_MAX_BITS; ++i) wd[i] = 0;
    if (r >= 0 && r < rows && w < cw) {
        float d = grid_step(__uint_as_float(*absmax_slot), bits);
        const float *src = W + (size_t)r * (size_t)cols;
        for (int b = 0; b < 32; ++b) {
            int c = w * 32 + b;
            if (c >= cols) break;
            uint32_t u = (uint32_t)quantize_code(src[c], d, bits);
#pragma unroll
            for (int i = 0; i < PB_MAX_BITS; ++i)
                if (i < bits) wd[i] |= ((u >> (bits - 1 - i)) & 1u) << b;
        }
    }
#pragma unroll
    for (int i = 0; i < PB_MAX_BITS; ++i)
        if (i < bits) packed[word_index(layout, cwp, layer_words, i, pr, w)] = wd[i];
}

// reads max|W| from scales[0] (where k_absmax left it) and writes the layer scales
__global__ void k_scales(float *scales, int bits)
{
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    float d = grid_step(scales[0], bits);
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
        uint32_t word = packed[word_index(layout, cwp, layer_words, i, pr, c >> 5)];
        u |= ((word >> (c & 31)) & 1u) << (bits - 1 - i);
    }
    int32_t v = (int32_t)(u << (32 - bits)) >> (32 - bits);  // sign-extend the B-bit code
    q[idx] = v;
}

int launch_quantize_pack(const float *W, const Layout &L, uint32_t *packed, float *scales, hipStream_t st)
{
    size_t n = (size_t)L.rows * (size_t)L.cols;
    uint32_t *slot = reinterpret_cast<uint32_t *>(scales);
    hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, st, slot, (size_t)1, 0u);
    int blocks = (int)((n + 256 * 16 - 1) / (256 * 16));
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(k_absmax, dim3(blocks), dim3(256), 0, st, W, n, slot);
    size_t total = L.layer_words;
    hipLaunchKernelGGL(k_pack, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, W, L.layout, L.rows, L.cols,
                       L.bits, L.cw, L.cwp, L.rows_p, L.gate_h, L.layer_words, slot, packed);
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

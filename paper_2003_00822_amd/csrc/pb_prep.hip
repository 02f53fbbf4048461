// Run-time activation processing (Algorithm 2 of the paper, x_q = Int(x * 2^f);
// Section 3.3: "a multiplication and a cast"; Section 3.4: the bitwise matrix
// transpose that lays the bits of one plane next to each other for AND/popcount).
//
// One workgroup per activation vector.  A thread owns 32 consecutive columns:
// it converts them to fixed point and transposes the 32x32 bit matrix in
// registers, which yields one packed word of each of the 32 planes.  The
// workgroup also reduces the plane statistics that let the product kernel skip
// planes that carry no information: h = number of magnitude bits in use (planes
// h..31 all equal the sign plane, so together they weigh -2^h), and whether any
// value is negative.  Skipping them changes no result bit.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pb_kernels.h"

namespace pb {

// k-bit saturating, toward-zero conversion of p = x * 2^f; NaN -> 0.
__device__ __forceinline__ int32_t to_fixed(float p, float lim /* 2^(k-1) */, int32_t imax, int32_t imin)
{
    if (p != p) return 0;
    if (p >= lim) return imax;
    if (p <= -lim) return imin;
    return (int32_t)p;
}

// In-register transpose of a 32x32 bit matrix: on return bit b of a[j] is what bit j of a[b] was.
__device__ __forceinline__ void transpose32(uint32_t (&a)[32])
{
#pragma unroll
    for (int j = 16; j != 0; j >>= 1) {
        // m selects, in every group of 2j bits, the low j bits
        uint32_t m = 0xFFFFFFFFu / ((1u << j) + 1u);
#pragma unroll
        for (int k = 0; k < 32; ++k) {
            if ((k & j) == 0) {
                uint32_t t = ((a[k] >> j) ^ a[k + j]) & m;
                a[k] ^= t << j;
                a[k + j] ^= t;
            }
        }
    }
}

__global__ __launch_bounds__(256) void k_prep(const float *__restrict__ X0, int cols0, const float *__restrict__ X1,
                                              int cols1, int cw, int cwp, float fscale, float lim, int32_t imax,
                                              int32_t imin, uint32_t *__restrict__ planes, int *__restrict__ meta,
                                              int32_t *__restrict__ xq_out)
{
    __shared__ uint32_t s_mag, s_any;
    const int n = blockIdx.x;
    const int C = cols0 + cols1;
    if (threadIdx.x == 0) { s_mag = 0; s_any = 0; }
    __syncthreads();
    const float *x0 = X0 + (size_t)n * cols0;
    const float *x1 = X1 ? X1 + (size_t)n * cols1 : nullptr;
    uint32_t *pl = planes + (size_t)n * 32 * (size_t)cwp;
    uint32_t mag = 0, any = 0;
    for (int w = threadIdx.x; w < cwp; w += blockDim.x) {
        uint32_t a[32];
#pragma unroll
        for (int b = 0; b < 32; ++b) {
            int c = w * 32 + b;
            float v = 0.0f;
            if (c < cols0) v = x0[c];
            else if (c < C) v = x1[c - cols0];
            int32_t xq = to_fixed(v * fscale, lim, imax, imin);
            if (xq_out && c < C) xq_out[(size_t)n * C + c] = xq;
            a[b] = (uint32_t)xq;
            mag |= (uint32_t)(xq ^ (xq >> 31));
            any |= (uint32_t)xq;
        }
        transpose32(a);
#pragma unroll
        for (int j = 0; j < 32; ++j) pl[(size_t)j * cwp + w] = a[j];
    }
    for (int off = 32; off > 0; off >>= 1) {
        mag |= (uint32_t)__shfl_xor((int)mag, off, 64);
        any |= (uint32_t)__shfl_xor((int)any, off, 64);
    }
    if ((threadIdx.x & 63) == 0) { atomicOr(&s_mag, mag); atomicOr(&s_any, any); }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t mg = s_mag;
        int h = mg ? 32 - __clz((int)mg) : 0;   // magnitude planes 0..h-1; plane h is the sign plane
        int neg = (int)(s_any >> 31);
        int nplanes = neg ? h + 1 : h;          // planes that must be multiplied
        int *mt = meta + (size_t)n * kMetaInts;
        mt[0] = h;
        mt[1] = neg;
        mt[2] = (nplanes + 3) >> 2;             // passes of 4 planes
        mt[3] = nplanes;
    }
}

int launch_prep(const float *X0, int cols0, const float *X1, int cols1, int batch, const Layout &L, int frac_bits,
                int act_bits, uint32_t *planes, int *meta, int32_t *xq_out, hipStream_t st)
{
    float fscale = ldexpf(1.0f, frac_bits);
    float lim = ldexpf(1.0f, act_bits - 1);
    int32_t imax = (act_bits == 32) ? INT32_MAX : (int32_t)((1u << (act_bits - 1)) - 1u);
    int32_t imin = (act_bits == 32) ? INT32_MIN : -(int32_t)(1u << (act_bits - 1));
    hipLaunchKernelGGL(k_prep, dim3(batch), dim3(256), 0, st, X0, cols0, X1, cols1, L.cw, L.cwp, fscale, lim, imax,
                       imin, planes, meta, xq_out);
    return (int)hipGetLastError();
}

}  // namespace pb

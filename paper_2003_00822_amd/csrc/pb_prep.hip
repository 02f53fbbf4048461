// Run-time activation processing (Algorithm 2 of the paper, x_q = Int(x * 2^f);
// Section 3.3: "a multiplication and a cast"; Section 3.4: the bitwise matrix
// transpose that lays the bits of one plane next to each other for AND/popcount).
//
// A workgroup of 4 waves owns 256 consecutive columns of one activation vector, a
// lane one column.  The transpose is the wave64 ballot: bit j of the 64 lanes'
// fixed-point values IS two packed words of plane j; lane j keeps ballot j and
// stores it.  32 columns groups of a vector run in parallel on
// different CUs, so the step is launch-latency bound, not compute bound.
// Every workgroup also converts the whole vector once (it is a few KB, coalesced)
// to reduce the plane statistics that let the product kernel skip planes carrying
// no information: h = number of magnitude bits in use (planes h..31 all equal the
// sign plane and together weigh -2^h) and whether any value is negative.  Doing
// that per workgroup avoids any cross-workgroup reduction or second launch;
// skipping those planes changes no result bit.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pb_kernels.h"

namespace pb {

// k-bit saturating, toward-zero conversion of p = x * 2^f; NaN -> 0.  lim = 2^(k-1), lim_below = the largest
// float below it.  Branch-free: clamp into the range where the cast is defined, then patch the top end and NaN
// (the bottom end, -2^(k-1), converts exactly).
__device__ __forceinline__ int32_t to_fixed(float p, float lim, float lim_below, int32_t imax)
{
    const float pc = fminf(fmaxf(p, -lim), lim_below);
    int32_t r = (int32_t)pc;
    r = (p >= lim) ? imax : r;
    return (p != p) ? 0 : r;
}

__global__ __launch_bounds__(256) void k_prep(const float *__restrict__ X0, int cols0, const float *__restrict__ X1,
                                              int cols1, int cwp, float fscale, float lim, float lim_below,
                                              int32_t imax, uint32_t *__restrict__ planes, int *__restrict__ meta,
                                              int32_t *__restrict__ xq_out)
{
    __shared__ uint32_t s_mag, s_any;
    const int n = blockIdx.y;
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int C = cols0 + cols1;
    if (tid == 0) { s_mag = 0; s_any = 0; }
    __syncthreads();
    const float *x0 = X0 + (size_t)n * cols0;
    const float *x1 = X1 ? X1 + (size_t)n * cols1 : nullptr;

    auto fetch = [&](int c) -> float {
        float v = 0.0f;
        if (c < cols0) v = x0[c];
        else if (c < C) v = x1[c - cols0];
        return v;
    };
    // this lane's own column first, then the whole vector, 8 x 256 columns at a time (independent loads in flight)
    const float v_own = fetch((b << 8) + tid);
    uint32_t mag = 0, any = 0;
    const int chunks = (C + 255) >> 8;
    for (int k0 = 0; k0 < chunks; k0 += 8) {
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = fetch(((k0 + j) << 8) + tid);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int32_t xq = to_fixed(v[j] * fscale, lim, lim_below, imax);
            mag |= (uint32_t)(xq ^ (xq >> 31));
            any |= (uint32_t)xq;
        }
    }
    const int32_t mine = to_fixed(v_own * fscale, lim, lim_below, imax);
    const int c_own = (b << 8) + tid;
    if (xq_out && c_own < C) xq_out[(size_t)n * C + c_own] = mine;

    // bitwise transpose of this wave's 64 columns: ballot j = words (2g, 2g+1) of plane j
    // (a select per plane rather than v_writelane: the compiler then inserts the wait states that a VALU-written
    // SGPR needs before a lane-indexed write reads it)
    uint32_t lo = 0, hi = 0;
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        const unsigned long long bal = __ballot((mine >> j) & 1);
        lo = (lane == j) ? (uint32_t)bal : lo;
        hi = (lane == j) ? (uint32_t)(bal >> 32) : hi;
    }
    const int word0 = 2 * (4 * b + wave);
    if (lane < 32 && word0 < cwp) {
        uint32_t *dst = planes + ((size_t)n * 32 + lane) * (size_t)cwp + word0;
        *reinterpret_cast<uint2 *>(dst) = make_uint2(lo, hi);
    }

    for (int off = 32; off > 0; off >>= 1) {
        mag |= (uint32_t)__shfl_xor((int)mag, off, 64);
        any |= (uint32_t)__shfl_xor((int)any, off, 64);
    }
    if (lane == 0) { atomicOr(&s_mag, mag); atomicOr(&s_any, any); }
    __syncthreads();
    if (b == 0 && tid == 0) {
        const uint32_t mg = s_mag;
        const int h = mg ? 32 - __clz((int)mg) : 0;   // magnitude planes 0..h-1; plane h is the sign plane
        const int neg = (int)(s_any >> 31);
        const int nplanes = neg ? h + 1 : h;          // planes that must be multiplied
        int *mt = meta + (size_t)n * kMetaInts;
        mt[0] = h;
        mt[1] = neg;
        mt[2] = (nplanes + 3) >> 2;                   // passes of 4 planes
        mt[3] = nplanes;
    }
}

int launch_prep(const float *X0, int cols0, const float *X1, int cols1, int batch, const Layout &L, int frac_bits,
                int act_bits, uint32_t *planes, int *meta, int32_t *xq_out, hipStream_t st)
{
    float fscale = ldexpf(1.0f, frac_bits);
    float lim = ldexpf(1.0f, act_bits - 1);
    int32_t imax = (act_bits == 32) ? INT32_MAX : (int32_t)((1u << (act_bits - 1)) - 1u);
    float lim_below = nextafterf(lim, 0.0f);
    hipLaunchKernelGGL(k_prep, dim3(L.cwp / 8, batch), dim3(256), 0, st, X0, cols0, X1, cols1, L.cwp, fscale, lim,
                       lim_below, imax, planes, meta, xq_out);
    return (int)hipGetLastError();
}

}  // namespace pb

// Calibration loops for the roofline figures of the benchmark (not a step of the method and not part of the
// product library: built into a library of its own, which only bench.py and its test load): what rate the FP4
// matrix instruction of the product kernel reaches on this chip by itself, and with the vector-ALU work that
// the kernel does beside it (expansion of one packed weight word per step, digit weighting + conversion + LDS
// atomic per chain of four steps).  The operands are constants; nothing is read from or written to memory but
// one float per workgroup.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pb {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

// MODE 0: four independent instructions per step.  MODE 1: + the seven-operation expansion of a weight word per
// step.  MODE 2: + per chain of four steps and per accumulator four FMAs, a conversion and an LDS atomic (the
// kernel's epilogue).
template <int MODE>
__global__ __launch_bounds__(512) void k_calib_mfma(int iters, float *out)
{
    constexpr int NV = 4;
    __shared__ int sums[64];
    const int lane = threadIdx.x & 63;
    if (threadIdx.x < 64) sums[threadIdx.x] = 0;
    __syncthreads();
    v8i a[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) a[v] = v8i{0x01230123 + v, 0x32103210, 0x11223300, 0x00112233, 0, 0, 0, 0};
    v8i b = {0x44444444, 0x04040404, 0x40404040, 0x44004400, 0, 0, 0, 0};
    v4f c[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) c[v] = v4f{0.f, 0.f, 0.f, 0.f};
    uint32_t w = 0x9E3779B9u * (uint32_t)(lane + 1);
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if (MODE >= 1) {
                asm volatile("" : "+v"(w));   // a fresh word as far as the compiler knows
                b[0] = (int)((w << 2) & 0x44444444u); b[1] = (int)((w << 1) & 0x44444444u);
                b[2] = (int)(w & 0x44444444u);        b[3] = (int)((w >> 1) & 0x44444444u);
            }
#pragma unroll
            for (int v = 0; v < NV; ++v)
                c[v] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[v], b, c[v], 4, 4, 0, 0x7F, 0, 0x7F);
        }
        if (MODE >= 2) {
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const float f = c[v][0] + c[v][1] * 4.0f + c[v][2] * 16.0f + c[v][3] * 64.0f;
                atomicAdd(&sums[lane], (int)f);
                c[v] = v4f{0.f, 0.f, 0.f, 0.f};
            }
        }
    }
    float s = (float)w;
#pragma unroll
    for (int v = 0; v < NV; ++v) s += c[v][0] + c[v][1] + c[v][2] + c[v][3];
    __syncthreads();
    if (threadIdx.x == 0) out[blockIdx.x] = s + (float)sums[0];
}

}  // namespace pb

// `workgroups` workgroups of 512 threads (two waves per SIMD), 16 * iters matrix instructions (65536 flop each) per
// wave.  mode 0: the instructions alone; 1: with the expansion of one packed weight word per four instructions; 2:
// also with an epilogue (digit weighting, conversion, LDS atomic) per chain of four.  out: [workgroups] fp32 on the
// device, written (a checksum that keeps the loop alive).  Returns 0, 1 for arguments out of range (mode outside
// 0..2, iters outside 1..2^20, workgroups outside 1..65536, a null pointer: nothing is launched), 2 if the launch failed.
extern "C" int pb_calib_mfma(int mode, int iters, int workgroups, float *out, void *stream)
{
    if (mode < 0 || mode > 2 || iters < 1 || iters > (1 << 20) || workgroups < 1 || workgroups > 65536 || !out)
        return 1;
    void (*fn)(int, float *) = mode == 0   ? pb::k_calib_mfma<0>
                               : mode == 1 ? pb::k_calib_mfma<1>
                                           : pb::k_calib_mfma<2>;
    hipLaunchKernelGGL(fn, dim3((unsigned)workgroups), dim3(512), 0, static_cast<hipStream_t>(stream), iters, out);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

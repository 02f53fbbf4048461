// LSTM cell pointwise step on the gate pre-activations produced by the quantized
// product (Sections 4.2-4.3 of the paper: the LSTM's linear maps are quantized,
// nonlinearities stay in full precision).  Standard cell, gate order
// (input, forget, cell, output) along the 4H rows of the fused gate matrix.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pb_kernels.h"

namespace pb {

__global__ __launch_bounds__(256) void k_lstm_pointwise(const float *__restrict__ gates, const float *__restrict__ bias,
                                                        const float *__restrict__ c_prev, int H, int batch,
                                                        float *__restrict__ h_out, float *__restrict__ c_out)
{
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= H * batch) return;
    int n = idx / H, u = idx - n * H;
    const float *g = gates + (size_t)n * 4 * H;
    float gi = g[u], gf = g[H + u], gg = g[2 * H + u], go = g[3 * H + u];
    if (bias) { gi += bias[u]; gf += bias[H + u]; gg += bias[2 * H + u]; go += bias[3 * H + u]; }
    float cn = sigmoid_f(gf) * c_prev[idx] + sigmoid_f(gi) * tanhf(gg);
    float hn = sigmoid_f(go) * tanhf(cn);
    c_out[idx] = cn;
    h_out[idx] = hn;
}

__global__ __launch_bounds__(256) void k_bias_act(float *__restrict__ Y, const float *__restrict__ bias, int relu,
                                                  int rows, int total)
{
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    float y = Y[idx];
    if (bias) y += bias[idx % rows];
    if (relu) y = fmaxf(y, 0.0f);
    Y[idx] = y;
}

int launch_bias_act(float *Y, const float *bias, int relu, int rows, int batch, hipStream_t st)
{
    int total = rows * batch;
    hipLaunchKernelGGL(k_bias_act, dim3((total + 255) / 256), dim3(256), 0, st, Y, bias, relu, rows, total);
    return (int)hipGetLastError();
}

int launch_lstm_pointwise(const float *gates, const float *bias, const float *c_prev, int H, int batch, float *h_out,
                          float *c_out, hipStream_t st)
{
    int total = H * batch;
    hipLaunchKernelGGL(k_lstm_pointwise, dim3((total + 255) / 256), dim3(256), 0, st, gates, bias, c_prev, H, batch,
                       h_out, c_out);
    return (int)hipGetLastError();
}

}  // namespace pb

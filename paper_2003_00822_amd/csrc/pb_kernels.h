// Internal: launchers implemented by the .hip files of this library.
// Each returns a hipError_t value as int (0 = success); arguments are validated by the caller.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pb_layout.h"

namespace pb {

// pb_quantize.hip
int launch_quantize_pack(const float *W, const Layout &L, int quantizer, uint32_t *packed, float *scales,
                         hipStream_t st);
int launch_unpack(const uint32_t *packed, const Layout &L, int32_t *q, hipStream_t st);

// pb_prep.hip: fp32 activations -> fixed point -> bit planes + plane statistics.
// Row n of the activations is the concatenation [X0[n][0..cols0) ; X1[n][0..cols1)] (X1 may be null with cols1 = 0).
int launch_prep(const float *X0, int cols0, const float *X1, int cols1, int batch, const Layout &L, int frac_bits,
                int act_bits, uint32_t *planes, int *meta, int32_t *xq_out, hipStream_t st);

// pb_matvec.hip: AND + popcount product against register-resident planes, one launch for all bitlayers.
// Exactly one of Y / A is non-null.
int launch_matvec(const uint32_t *packed, const float *scales, const Layout &L, int bits_used, int frac_bits,
                  const uint32_t *planes, const int *meta, int batch, float *Y, long long *A, hipStream_t st);

// pb_mfma.hip: the whole of Algorithm 2 in one launch on the matrix cores (the tiled layouts).  Activations come
// from X0 / X1 (converted and bit-transposed inside the kernel) or, if `planes` is non-null, from bit planes that
// launch_prep left in memory.  Exactly one of Y / A is non-null.
// What follows the product in the same launch: bias and ReLU before the store of Y, or (PB_LAYOUT_TILE16_GATES_V1
// only) the LSTM cell update, which writes h_out / c_out [batch][H] instead of Y.
struct Epilogue {
    const float *bias = nullptr;   // [rows] or null
    int relu = 0;
    const float *c_prev = nullptr; // non-null: fused LSTM cell
    float *h_out = nullptr, *c_out = nullptr;
};
int launch_mfma(const uint32_t *packed, const float *scales, const Layout &L, int bits_used, int frac_bits,
                int act_bits, const float *X0, int cols0, const float *X1, int cols1, const uint32_t *planes,
                int batch, float *Y, long long *A, bool pairs_out, const Epilogue &ep, hipStream_t st);

// logistic function of the LSTM gates in the stand-alone cell update (the fused one evaluates 0.5 tanh(v / 2) + 0.5,
// the same function, side by side with the tanh of the fourth gate)
__device__ __forceinline__ float sigmoid_f(float v) { return 1.0f / (1.0f + expf(-v)); }

// pb_lstm.hip: y = act(y + bias) in place, for the layout whose product kernel has no fused epilogue
int launch_bias_act(float *Y, const float *bias, int relu, int rows, int batch, hipStream_t st);

// pb_lstm.hip: gate nonlinearities and state update on the gate pre-activations.
int launch_lstm_pointwise(const float *gates, const float *bias, const float *c_prev, int H, int batch, float *h_out,
                          float *c_out, hipStream_t st);

}  // namespace pb

// The arithmetic of the recurrent cells (Section 3.1: an RNN step is a matrix-vector product; what follows it is
// elementwise).  One definition for every kernel that applies a cell -- the stand-alone cell kernels, the one-step
// kernels with the cell in their epilogue, and the whole-sequence kernel -- with the multiply-adds spelled out, so
// that all of them round alike and a sequence computed either way agrees bit for bit.
#pragma once
#include <hip/hip_runtime.h>

#include "grim_bcr.h"

namespace grim {

__device__ __forceinline__ float rnn_sigmoid(float v) { return 1.0f / (1.0f + expf(-v)); }

// round to nearest even; NaN stays NaN
__device__ __forceinline__ unsigned short rnn_f32_to_bf16(float f) {
    unsigned int u = __builtin_bit_cast(unsigned int, f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

__device__ __forceinline__ void rnn_store_h(void *h, int hdt, int64_t at, float v) {
    if (hdt == GRIM_F32) static_cast<float *>(h)[at] = v;
    else if (hdt == GRIM_F16) static_cast<_Float16 *>(h)[at] = (_Float16)v;
    else static_cast<unsigned short *>(h)[at] = rnn_f32_to_bf16(v);
}

// LSTM: gate pre-activations with their bias already added; c is updated, the new h returned
//     i, f, o = sigmoid(.), g = tanh(.), c <- f * c + i * g, h = o * tanh(c)
__device__ __forceinline__ float lstm_cell_apply(float pi, float pf, float pg, float po, float &c) {
    const float gi = rnn_sigmoid(pi);
    const float gf = rnn_sigmoid(pf);
    const float gg = tanhf(pg);
    const float go = rnn_sigmoid(po);
    c = __builtin_fmaf(gf, c, gi * gg);
    return go * tanhf(c);
}

// GRU: input-side (i*) and hidden-side (h*) pre-activations with their biases added; returns the new h
//     r = sigmoid(ir + hr), z = sigmoid(iz + hz), n = tanh(in + r * hn), h' = (1 - z) * n + z * h
__device__ __forceinline__ float gru_cell_apply(float ir, float iz, float in, float hr, float hz, float hn, float h) {
    const float r = rnn_sigmoid(ir + hr);
    const float z = rnn_sigmoid(iz + hz);
    const float n = tanhf(__builtin_fmaf(r, hn, in));
    return __builtin_fmaf(z, h, (1.0f - z) * n);
}

}  // namespace grim

// The arithmetic of the recurrent cells (Section 3.1: an RNN step is a matrix-vector product; what follows it is
// elementwise).  One definition for every kernel that applies a cell -- the stand-alone cell kernels, the one-step
// kernels with the cell in their epilogue, and the whole-sequence kernel -- with the multiply-adds spelled out, so
// that all of them round alike and a sequence computed either way agrees bit for bit.
#pragma once
#include <hip/hip_runtime.h>

#include "grim_bcr.h"

namespace grim {

// The two activations on the hardware's exponential and reciprocal (v_exp_f32, v_rcp_f32: 1 ulp each; overflow gives
// infinity and its reciprocal 0, so both saturate by themselves): a cell is a dependent chain of five of them in one
// thread per hidden unit, at the end of a step that everything else waits for, and the library's expf, tanhf and the
// correctly rounded division are four times the instructions.  Absolute error below 2e-7 (tanh near 0: the
// difference 1 - 2 / (e + 1) cancels, so small results carry that absolute, not a relative, error).
__device__ __forceinline__ float rnn_sigmoid(float v) {
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(v * -1.44269504088896340736f));
}
__device__ __forceinline__ float rnn_tanh(float v) {
    return __builtin_fmaf(-2.0f, __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(v * 2.88539008177792681472f)), 1.0f);
}

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
    const float gg = rnn_tanh(pg);
    const float go = rnn_sigmoid(po);
    c = __builtin_fmaf(gf, c, gi * gg);
    float h = go * rnn_tanh(c);
    asm volatile("" : "+v"(h));       // h exists as an fp32 value: a later rounding to 16 bits is a step of its own in every kernel
    return h;
}

// GRU: input-side (i*) and hidden-side (h*) pre-activations with their biases added; returns the new h
//     r = sigmoid(ir + hr), z = sigmoid(iz + hz), n = tanh(in + r * hn), h' = (1 - z) * n + z * h
__device__ __forceinline__ float gru_cell_apply(float ir, float iz, float in, float hr, float hz, float hn, float h) {
    const float r = rnn_sigmoid(ir + hr);
    const float z = rnn_sigmoid(iz + hz);
    const float n = rnn_tanh(__builtin_fmaf(r, hn, in));
    float hn2 = __builtin_fmaf(z, h, (1.0f - z) * n);
    asm volatile("" : "+v"(hn2));     // (as in the LSTM cell: no rounding to 16 bits fused into the last operation)
    return hn2;
}

}  // namespace grim

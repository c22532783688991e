// Recurrent cells around the gate products.
//
// LSTM cell (Section 3.1: the gate matrices of an RNN layer are one
// matrix-vector product per time step; Section 6 evaluates RNNs end to end).
//
// The BCR product y = [W_ih | W_hh] * [x; h] delivers the four gate pre-activations stacked as
// rows [0, H) input gate, [H, 2H) forget gate, [2H, 3H) cell candidate, [3H, 4H) output gate.
// This kernel is the elementwise rest of the step:
//     i = sigmoid(y_i + b_i)   f = sigmoid(y_f + b_f)   g = tanh(y_g + b_g)   o = sigmoid(y_o + b_o)
//     c' = f * c + i * g        h' = o * tanh(c')
// c stays fp32 and is updated in place; h' is written in the matrix's element type straight into
// the lower part of the next step's input vector [x; h], and optionally as fp32 as well.
#include <hip/hip_runtime.h>

#include "bcr_matrix.hpp"
#include "rnn_cell.hpp"

namespace grim {

struct LstmParams {
    const float *gates;
    const float *bias;
    float *c;
    void *h;
    float *h32;
    int64_t ldg, ldc, ldh, ldh32, H;
    int32_t batch, dtype;
};

__global__ void __launch_bounds__(256) lstm_cell_kernel(LstmParams p) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= p.H * p.batch) return;
    const int64_t r = e / p.batch;
    const int b = (int)(e - r * p.batch);
    const float bi = p.bias ? p.bias[r] : 0.f, bf = p.bias ? p.bias[p.H + r] : 0.f;
    const float bg = p.bias ? p.bias[2 * p.H + r] : 0.f, bo = p.bias ? p.bias[3 * p.H + r] : 0.f;
    float c = p.c[r * p.ldc + b];
    const float h = lstm_cell_apply(p.gates[r * p.ldg + b] + bi, p.gates[(p.H + r) * p.ldg + b] + bf,
                                    p.gates[(2 * p.H + r) * p.ldg + b] + bg, p.gates[(3 * p.H + r) * p.ldg + b] + bo, c);
    p.c[r * p.ldc + b] = c;
    if (p.h32) p.h32[r * p.ldh32 + b] = h;
    if (p.h) rnn_store_h(p.h, p.dtype, r * p.ldh + b, h);
}

// GRU cell (Section 6.1: the evaluated RNN is a two-layer GRU; Section 6.3 times it).  Two products feed it, gi = W_i x and gh = W_h h,
// each with its gate rows stacked reset, update, candidate; the reset gate scales the hidden-side
// candidate product, which is why the two cannot be one product of a stacked matrix:
//     r = sigmoid(gi_r + bi_r + gh_r + bh_r)        z = sigmoid(gi_z + bi_z + gh_z + bh_z)
//     n = tanh(gi_n + bi_n + r * (gh_n + bh_n))     h' = (1 - z) * n + z * h
// The state h stays fp32 and is updated in place; h' is also written in the matrix's element type,
// the form the next step's hidden-side product reads.
struct GruParams {
    const float *gi, *gh;
    const float *bias_i, *bias_h;
    float *h32;
    void *h;
    int64_t ldgi, ldgh, ldh32, ldh, H;
    int32_t batch, dtype;
};

__global__ void __launch_bounds__(256) gru_cell_kernel(GruParams p) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= p.H * p.batch) return;
    const int64_t j = e / p.batch;
    const int b = (int)(e - j * p.batch);
    float pi[3], ph[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        pi[k] = p.gi[(k * p.H + j) * p.ldgi + b] + (p.bias_i ? p.bias_i[k * p.H + j] : 0.f);
        ph[k] = p.gh[(k * p.H + j) * p.ldgh + b] + (p.bias_h ? p.bias_h[k * p.H + j] : 0.f);
    }
    const float h = gru_cell_apply(pi[0], pi[1], pi[2], ph[0], ph[1], ph[2], p.h32[j * p.ldh32 + b]);
    p.h32[j * p.ldh32 + b] = h;
    if (p.h) rnn_store_h(p.h, p.dtype, j * p.ldh + b, h);
}

grim_status launch_gru_cell(const float *gi, int64_t ldgi, const float *gh, int64_t ldgh, const float *bias_i,
                            const float *bias_h, float *h32, int64_t ldh32, void *h, int32_t dtype, int64_t ldh,
                            int64_t H, int32_t batch, hipStream_t stream) {
    GruParams p{gi, gh, bias_i, bias_h, h32, h, ldgi, ldgh, ldh32, ldh, H, batch, dtype};
    const int64_t nwg = (H * batch + 255) / 256;
    if (nwg > 0x7fffffff) return GRIM_ERR_SHAPE;
    hipLaunchKernelGGL(gru_cell_kernel, dim3((unsigned)nwg), dim3(256), 0, stream, p);
    return hipGetLastError() == hipSuccess ? GRIM_OK : GRIM_ERR_DEVICE;
}

grim_status launch_lstm_cell(const float *gates, int64_t ldg, const float *bias, float *c, int64_t ldc, void *h,
                             int32_t dtype, int64_t ldh, float *h32, int64_t ldh32, int64_t H, int32_t batch,
                             hipStream_t stream) {
    LstmParams p{gates, bias, c, h, h32, ldg, ldc, ldh, ldh32, H, batch, dtype};
    const int64_t n = H * batch;
    const int64_t nwg = (n + 255) / 256;
    if (nwg > 0x7fffffff) return GRIM_ERR_SHAPE;
    hipLaunchKernelGGL(lstm_cell_kernel, dim3((unsigned)nwg), dim3(256), 0, stream, p);
    return hipGetLastError() == hipSuccess ? GRIM_OK : GRIM_ERR_DEVICE;
}

}  // namespace grim

// SpMV / skinny SpMM kernel: y = W_bcr * x for 1..8 right-hand sides (Section 3.1: FC and
// RNN gate layers are matrix-vector products).
//
// The compact weights ARE the memory traffic here, so they are read exactly once, in
// their compact kept-rows x kept-columns form (Section 4.3), with 8 bytes of row / column
// bit masks per block as the only index data.  One workgroup owns one row strip.  Eight
// lanes share a block: lane i takes compact rows i, i + 8, ... and walks the row's kept
// columns, taking x from an LDS copy (every gathered x value is shared by all kept rows of
// the block -- the load-redundancy elimination of Section 4.4).  Per-block partial sums go
// to private LDS slots; one thread per (strip row, right-hand side) then adds the partials
// of the blocks that keep its row in ascending column-block order: fixed order, no atomics.
#include <hip/hip_runtime.h>

#include "bcr_matrix.hpp"

namespace grim {

struct GemvParams {
    const GemvDesc *table;   // device table (batched launch) or nullptr
    GemvDesc single;
    int32_t BR, BC, nbc, K;
    int32_t ukr, ukc;        // uniform kept counts or -1
    const void *x;
    float *y;
    int64_t x_stride, y_stride, ldx, ldy;
    int32_t xvec16;          // x is contiguous and 16-byte aligned: copy with 16-byte loads
};

template <int DT> struct GElem;
template <> struct GElem<GRIM_F32> { using type = float; };
template <> struct GElem<GRIM_F16> { using type = _Float16; };
template <> struct GElem<GRIM_BF16> { using type = unsigned short; };

template <int DT> __device__ __forceinline__ float g2f(typename GElem<DT>::type v);
template <> __device__ __forceinline__ float g2f<GRIM_F32>(float v) { return v; }
template <> __device__ __forceinline__ float g2f<GRIM_F16>(_Float16 v) { return (float)v; }
template <> __device__ __forceinline__ float g2f<GRIM_BF16>(unsigned short v) {
    return __builtin_bit_cast(float, (unsigned int)v << 16);
}

constexpr int kSlots = 32;      // blocks in flight per workgroup pass (8 lanes each)
constexpr int kRowsMax = 32;    // BR <= 32

template <int DT, int B, int VEC>
__global__ void __launch_bounds__(256) bcr_spmv(GemvParams p) {
    using T = typename GElem<DT>::type;
    struct __attribute__((aligned(sizeof(T) * VEC))) WVec { T v[VEC]; };
    extern __shared__ __attribute__((aligned(16))) char smem[];
    float *part = reinterpret_cast<float *>(smem);                        // [kSlots][kRowsMax][B]
    unsigned int *msk = reinterpret_cast<unsigned int *>(part + kSlots * kRowsMax * B);   // [kSlots]
    T *xs = reinterpret_cast<T *>(msk + kSlots);                          // [K][B]

    const int tid = threadIdx.x;
    const int64_t t = blockIdx.x;            // stored strip
    const int64_t mi = blockIdx.y;           // matrix of the group
    const GemvDesc d = p.table ? p.table[mi] : p.single;
    const T *W = static_cast<const T *>(d.weights);
    const T *x = static_cast<const T *>(p.x) + mi * p.x_stride;
    float *y = p.y + mi * p.y_stride;

    // x -> LDS, layout [k][b]
    const int nx = p.K * B;
    if (p.xvec16) {
        constexpr int PER = 16 / sizeof(T);
        const uint4 *src = reinterpret_cast<const uint4 *>(x);
        uint4 *dst = reinterpret_cast<uint4 *>(xs);
        for (int e = tid; e < nx / PER; e += 256) dst[e] = src[e];
    } else {
        for (int e = tid; e < nx; e += 256) xs[e] = x[(int64_t)(e / B) * p.ldx + (e % B)];
    }
    __syncthreads();

    const int bs = tid >> 3, i0 = tid & 7;
    const int r_out = tid / B, b_out = tid % B;      // reducer role: tid < BR * B
    float yacc = 0.f;

    for (int cbase = 0; cbase < p.nbc; cbase += kSlots) {
        const int c = cbase + bs;
        unsigned int rm = 0, cm = 0;
        if (c < p.nbc) {
            const int64_t blk = t * p.nbc + c;
            rm = d.masks[2 * blk];
            cm = d.masks[2 * blk + 1];
            const int kr = __builtin_popcount(rm), kc = __builtin_popcount(cm);
            const unsigned int woff = p.ukr >= 0 ? (unsigned int)blk * (unsigned int)(p.ukr * p.ukc) : d.woff[blk];
            const int xbase = c * p.BC;
            for (int i = i0; i < kr; i += 8) {
                const T *wr = W + woff + i * kc;
                float acc[B];
#pragma unroll
                for (int b = 0; b < B; ++b) acc[b] = 0.f;
                unsigned int m = cm;
                for (int j = 0; j < kc; j += VEC) {
                    const WVec wv = *reinterpret_cast<const WVec *>(wr + j);
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        const int col = __builtin_ctz(m);
                        m &= m - 1;
                        const float w = g2f<DT>(wv.v[v]);
                        const T *xp = xs + (xbase + col) * B;
#pragma unroll
                        for (int b = 0; b < B; ++b) acc[b] = __builtin_fmaf(w, g2f<DT>(xp[b]), acc[b]);
                    }
                }
#pragma unroll
                for (int b = 0; b < B; ++b) part[(bs * kRowsMax + i) * B + b] = acc[b];
            }
        }
        if (i0 == 0) msk[bs] = rm;
        __syncthreads();
        if (tid < p.BR * B) {
#pragma unroll 8
            for (int s = 0; s < kSlots; ++s) {
                const unsigned int m = msk[s];
                if ((m >> r_out) & 1u) {
                    const int i = __builtin_popcount(m & ((1u << r_out) - 1u));
                    yacc += part[(s * kRowsMax + i) * B + b_out];
                }
            }
        }
        __syncthreads();
    }
    if (tid < p.BR * B) {
        const int64_t row = (int64_t)d.strip_order[t] * p.BR + r_out;
        y[row * p.ldy + b_out] = yacc;
    }
}

template <int DT, int B>
static grim_status launch_vec(const GemvParams &p, int vec, dim3 grid, size_t lds, hipStream_t stream) {
#define GRIM_GEMV(V)                                                                                          \
    {                                                                                                         \
        auto kern = bcr_spmv<DT, B, V>;                                                                       \
        if (lds > 64 * 1024 &&                                                                                \
            hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) { \
            (void)hipGetLastError();                                                                          \
            return GRIM_ERR_DEVICE;                                                                           \
        }                                                                                                     \
        hipLaunchKernelGGL(kern, grid, dim3(256), lds, stream, p);                                            \
        return hipGetLastError() == hipSuccess ? GRIM_OK : GRIM_ERR_DEVICE;                                   \
    }
    if (vec >= 8 && sizeof(typename GElem<DT>::type) == 2) GRIM_GEMV(8)
    if (vec >= 4) GRIM_GEMV(4)
    if (vec >= 2) GRIM_GEMV(2)
    GRIM_GEMV(1)
#undef GRIM_GEMV
}

template <int DT>
static grim_status launch_batch(const GemvParams &p, int batch, int vec, dim3 grid, size_t lds, hipStream_t stream) {
    switch (batch) {
        case 1: return launch_vec<DT, 1>(p, vec, grid, lds, stream);
        case 2: return launch_vec<DT, 2>(p, vec, grid, lds, stream);
        case 3: return launch_vec<DT, 3>(p, vec, grid, lds, stream);
        case 4: return launch_vec<DT, 4>(p, vec, grid, lds, stream);
        case 5: return launch_vec<DT, 5>(p, vec, grid, lds, stream);
        case 6: return launch_vec<DT, 6>(p, vec, grid, lds, stream);
        case 7: return launch_vec<DT, 7>(p, vec, grid, lds, stream);
        case 8: return launch_vec<DT, 8>(p, vec, grid, lds, stream);
    }
    return GRIM_ERR_SHAPE;
}

grim_status launch_spmv(const GemvDesc *table, const GemvDesc &single, int32_t count, int64_t M, int64_t K, int32_t BR,
                        int32_t BC, int32_t dtype, int32_t ukr, int32_t ukc, int32_t vec, const void *x, int64_t x_stride,
                        int32_t batch, int64_t ldx, float *y, int64_t y_stride, int64_t ldy, hipStream_t stream) {
    if (BR > kRowsMax || BC > 32 || batch < 1 || batch > 8) return GRIM_ERR_UNSUPPORTED;
    const int esz = dtype_size(dtype);
    const int64_t nbr = M / BR;
    if (nbr > 0x7fffffff || count > 65535) return GRIM_ERR_SHAPE;
    GemvParams p;
    p.table = table;
    p.single = single;
    p.BR = BR; p.BC = BC; p.nbc = (int32_t)(K / BC); p.K = (int32_t)K;
    p.ukr = ukr; p.ukc = ukc;
    p.x = x; p.y = y; p.x_stride = x_stride; p.y_stride = y_stride; p.ldx = ldx; p.ldy = ldy;
    const bool contiguous = ldx == batch && reinterpret_cast<uintptr_t>(x) % 16 == 0 &&
                            (K * batch * esz) % 16 == 0 && (count == 1 || (x_stride * esz) % 16 == 0);
    p.xvec16 = contiguous ? 1 : 0;
    const size_t lds = (size_t)kSlots * kRowsMax * batch * 4 + kSlots * 4 + (((size_t)K * batch * esz + 15) & ~size_t(15));
    if (lds > 160 * 1024) return GRIM_ERR_UNSUPPORTED;
    dim3 grid((unsigned)nbr, (unsigned)count);
    switch (dtype) {
        case GRIM_F32: return launch_batch<GRIM_F32>(p, batch, vec, grid, lds, stream);
        case GRIM_F16: return launch_batch<GRIM_F16>(p, batch, vec, grid, lds, stream);
        case GRIM_BF16: return launch_batch<GRIM_BF16>(p, batch, vec, grid, lds, stream);
    }
    return GRIM_ERR_DTYPE;
}

}  // namespace grim

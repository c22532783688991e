// Declarations shared by the SpMV kernels and the recurrent-sequence kernel: launch parameters, element types,
// the LDS placement of a strip's blocks, and the cell arithmetic.
#pragma once
#include <hip/hip_runtime.h>

#include "bcr_matrix.hpp"
#include "rnn_cell.hpp"

namespace grim {

struct GemvParams {
    const GemvDesc *table;   // device table (batched launch) or nullptr
    GemvDesc single;         // no table: matrix 0 ...
    GemvDesc second;         // ... and matrix 1 of a two-matrix launch
    int32_t BR, BC, nbc, K;
    int32_t nbr_total;       // row strips of the matrix
    int32_t ukr, ukc;        // uniform kept counts or -1
    int32_t lpb_shift;       // log2(lanes per block), 2..5
    int32_t seg_blocks;      // column blocks per LDS segment (<= kSegMax)
    int32_t wbytes;          // LDS bytes reserved for a segment's weights
    int32_t krmax, kcmax;    // most rows / columns any block keeps
    const void *x;
    float *y;
    int64_t x_stride, y_stride, ldx, ldy;
    int32_t xvec16;          // x is contiguous and 16-byte aligned: copy with 16-byte loads
    int32_t sps;             // wave kernel: consecutive strips per wave
    int32_t wpg;             // one-column wave kernel without a cell: waves of a workgroup that take strips (1, 2 or 4)
    int32_t batch;           // right-hand sides (kernels that take it at run time)
    RnnCell cell;            // recurrent cell in the epilogue (wave-per-strip kernel, one right-hand side)
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

constexpr int kSegMax = 64;          // column blocks per segment at most
constexpr int kWLoads = 8;           // 16-byte weight loads per thread per segment (256 threads: 32 KB)
constexpr int kGemvWBytes = kWLoads * 256 * 16;

typedef unsigned int gu32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int gu32x2 __attribute__((ext_vector_type(2)));

// Pointers read out of a descriptor in memory carry no address space, and loads through them
// would be generic ("flat") loads, which also tick the counter that LDS traffic is waited on.
// Everything the descriptors point to is device global memory, so the kernels say so.
#define GRIM_GLOBAL __attribute__((address_space(1)))
struct GemvGlobal {
    const GRIM_GLOBAL char *weights;
    const GRIM_GLOBAL unsigned int *masks;
    const GRIM_GLOBAL unsigned int *woff;
    const GRIM_GLOBAL int *strip_order;
};
__device__ __forceinline__ GemvGlobal to_global(const GemvDesc &d) {
    GemvGlobal g;
    g.weights = (const GRIM_GLOBAL char *)d.weights;
    g.masks = (const GRIM_GLOBAL unsigned int *)d.masks;
    g.woff = (const GRIM_GLOBAL unsigned int *)d.woff;
    g.strip_order = (const GRIM_GLOBAL int *)d.strip_order;
    return g;
}

// position of the j-th (0-based) set bit of m; j < popcount(m)
__device__ __forceinline__ int nth_set_bit(unsigned int m, int j) {
    int pos = 0;
    int c = __builtin_popcount(m & 0xffffu);
    if (j >= c) { j -= c; m >>= 16; pos = 16; }
    c = __builtin_popcount(m & 0xffu);
    if (j >= c) { j -= c; m >>= 8; pos += 8; }
    c = __builtin_popcount(m & 0xfu);
    if (j >= c) { j -= c; m >>= 4; pos += 4; }
    c = __builtin_popcount(m & 0x3u);
    if (j >= c) { j -= c; m >>= 2; pos += 2; }
    if (j >= (int)(m & 1u)) pos += 1;
    return pos;
}

__host__ __device__ inline int gemv_xg_stride(int kcmax, int B) { return ((kcmax + 7) & ~7) * B; }

typedef _Float16 gh2 __attribute__((ext_vector_type(2)));
typedef __bf16 gb2 __attribute__((ext_vector_type(2)));


constexpr int kPartStride = 66;                    // floats per strip row of the partial table (wave-per-strip kernels)

// Wave-per-strip kernels, one right-hand side: lane l gathers the kept activations of column block l from the LDS copy of
// x.  Blocks of BC elements are a multiple of 16 bytes apart (32 fp16: 64 bytes), so the lanes of such a 2-byte read fall
// on every fourth, eighth or sixteenth bank only and take turns.  With 4 bytes of padding behind every block's part of
// x the blocks are an odd number of banks apart.  (Blocks whose size is no multiple of 16 bytes keep the plain layout:
// a 16-byte unit of the copy may not straddle two blocks.)  Elements of padding per block:
__host__ __device__ inline int exact_x_skew(int BC, int esz) { return (BC * esz) % 16 == 0 ? 4 / esz : 0; }

// Lanes read their blocks with 16-byte loads at a common offset from bases NV vectors apart;
// 16 such vectors span the LDS banks.  When NV shares a factor g with 16 the bases of 16
// neighbouring lanes fall on only 16/g distinct bank groups, so one vector of padding goes
// after every 16/g blocks, which shifts each run of 16/g lanes onto its own group.
__host__ __device__ constexpr int exact_pad_period(int nv) {
    int g = 1;
    while (g < 16 && nv % (g * 2) == 0) g *= 2;
    return g == 1 ? 0 : 16 / g;
}
__host__ __device__ constexpr int exact_region_vectors(int nv) {
    return 64 * nv + (exact_pad_period(nv) ? 64 / exact_pad_period(nv) : 0);
}


// CELL: 0 = the product alone; 1 = LSTM step, 2 = GRU step (see RnnCell): the workgroup's waves take the strips of
// one group of BR hidden units, and the cell is applied to their sums before anything is stored.
constexpr int exact_waves(int cell) { return cell == 2 ? 6 : 4; }

}  // namespace grim

// SpMM kernels for Y = W_bcr * X (Section 3.1: CONV as GEMM on the im2col matrix).
//
//  * bcr_spmm_fma  -- portable kernel on the vector ALUs.  Any element type, BR <= 64.
//    One wave owns one row strip x 64 columns of X and walks the strip's blocks in
//    ascending column-block order; every gathered X value is loaded once and reused
//    by all kept rows of the block (the load-redundancy elimination of Section 4.4,
//    here a consequence of treating the block as a small dense matrix).
//  * bcr_spmm_mma  -- matrix-core kernel for fp16 / bf16 with BR = 16 or 32.
//    A workgroup owns a tile of TN columns of X and a group of row strips.  Chunks of
//    consecutive X rows are staged in LDS once per workgroup (tiling, Section 4.4);
//    each wave gathers the rows its strip keeps with LDS transpose reads straight into
//    MFMA operand layout and multiplies them with pre-built weight fragments.  Strips
//    are visited in stored (work-sorted, Section 4.2) order so the waves of a
//    workgroup carry near-equal work.  Accumulation is fp32, order fixed, no atomics.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "bcr_matrix.hpp"

namespace grim {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef short i16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <int DT> struct Elem;
template <> struct Elem<GRIM_F32> { using type = float; };
template <> struct Elem<GRIM_F16> { using type = _Float16; };
template <> struct Elem<GRIM_BF16> { using type = unsigned short; };

template <int DT> __device__ __forceinline__ float to_f32(typename Elem<DT>::type v);
template <> __device__ __forceinline__ float to_f32<GRIM_F32>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<GRIM_F16>(_Float16 v) { return (float)v; }
template <> __device__ __forceinline__ float to_f32<GRIM_BF16>(unsigned short v) {
    return __builtin_bit_cast(float, (unsigned int)v << 16);
}

// ------------------------------------------------------------------------------------------
// portable FMA kernel
// ------------------------------------------------------------------------------------------
struct FmaParams {
    const int32_t *strip_order;
    const int32_t *row_ptr;
    const int32_t *col_ptr;
    const uint16_t *col_idx;
    const int64_t *blk_ptr;
    const uint64_t *rowmask;
    const void *weights;
    const void *X;
    float *Y;
    int64_t N, ldx, ldy;
    int32_t BR, BC;
    int64_t nbc;
};

template <int DT, int BRCAP>
__global__ void __launch_bounds__(64) bcr_spmm_fma(FmaParams p) {
    using T = typename Elem<DT>::type;
    const int64_t t = blockIdx.x;                        // stored strip
    const int64_t n = (int64_t)blockIdx.y * 64 + threadIdx.x;
    const bool live = n < p.N;
    const T *X = static_cast<const T *>(p.X);
    const T *W = static_cast<const T *>(p.weights);
    float acc[BRCAP];
#pragma unroll
    for (int r = 0; r < BRCAP; ++r) acc[r] = 0.f;
    for (int64_t c = 0; c < p.nbc; ++c) {
        const int64_t b = t * p.nbc + c;
        const uint64_t mask = p.rowmask[b];
        const int32_t cp0 = p.col_ptr[b];
        const int32_t kc = p.col_ptr[b + 1] - cp0;
        if (mask == 0 || kc == 0) continue;
        const T *wb = W + p.blk_ptr[b];
        for (int32_t j = 0; j < kc; ++j) {
            const int64_t k = c * p.BC + p.col_idx[cp0 + j];
            const float xv = live ? to_f32<DT>(X[k * p.ldx + n]) : 0.f;
            int32_t i = 0;
#pragma unroll
            for (int r = 0; r < BRCAP; ++r) {
                if ((mask >> r) & 1) {                  // same for the whole wave
                    acc[r] = __builtin_fmaf(to_f32<DT>(wb[(int64_t)i * kc + j]), xv, acc[r]);
                    ++i;
                }
            }
        }
    }
    if (live) {
        const int64_t row0 = (int64_t)p.strip_order[t] * p.BR;
#pragma unroll
        for (int r = 0; r < BRCAP; ++r)
            if (r < p.BR) p.Y[(row0 + r) * p.ldy + n] = acc[r];
    }
}

template <int DT>
static grim_status launch_fma_dt(const FmaParams &p, int32_t BR, int64_t nbr, hipStream_t stream) {
    if ((p.N + 63) / 64 > 65535 || nbr > 0x7fffffff) return GRIM_ERR_SHAPE;
    dim3 grid((unsigned)nbr, (unsigned)((p.N + 63) / 64));
    if (BR <= 16) hipLaunchKernelGGL((bcr_spmm_fma<DT, 16>), grid, dim3(64), 0, stream, p);
    else if (BR <= 32) hipLaunchKernelGGL((bcr_spmm_fma<DT, 32>), grid, dim3(64), 0, stream, p);
    else hipLaunchKernelGGL((bcr_spmm_fma<DT, 64>), grid, dim3(64), 0, stream, p);
    return hipGetLastError() == hipSuccess ? GRIM_OK : GRIM_ERR_DEVICE;
}

grim_status launch_spmm_fma(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, float *Y, int64_t ldy,
                            hipStream_t stream) {
    if (A->BR > 64) return GRIM_ERR_UNSUPPORTED;
    FmaParams p{A->dev.strip_order, A->dev.row_ptr, A->dev.col_ptr, A->dev.col_idx, A->dev.blk_ptr, A->dev.rowmask64,
                A->dev.weights, X, Y, N, ldx, ldy, A->BR, A->BC, A->nbc};
    switch (A->dtype) {
        case GRIM_F32: return launch_fma_dt<GRIM_F32>(p, A->BR, A->nbr, stream);
        case GRIM_F16: return launch_fma_dt<GRIM_F16>(p, A->BR, A->nbr, stream);
        case GRIM_BF16: return launch_fma_dt<GRIM_BF16>(p, A->BR, A->nbr, stream);
    }
    return GRIM_ERR_DTYPE;
}

// ------------------------------------------------------------------------------------------
// matrix-core kernel
// ------------------------------------------------------------------------------------------
struct MmaParams {
    const uint16_t *afrag;
    const uint16_t *kidx;
    const int32_t *kstep_ptr;
    const int32_t *strip_order;
    const unsigned short *X;
    float *Y;
    int64_t N, ldx, ldy;
    int32_t K, nbr, nchunks, chunk_rows;
    int32_t ntiles, ngroups;
    int32_t xvec;   // widest aligned vector (elements: 8, 4, 2 or 1) for rows of X
    int32_t yvec;   // 4 when rows of Y allow aligned float4 stores, else 1
};

template <bool BF16>
__device__ __forceinline__ f32x4 mfma16(i16x8 a, i16x8 b, f32x4 c) {
    if constexpr (BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
template <bool BF16>
__device__ __forceinline__ f32x16 mfma32(i16x8 a, i16x8 b, f32x16 c) {
    if constexpr (BF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// LDS transpose read: the 16 lanes of a block each name 8 bytes (4 values along n of one
// staged row); lane i of the block receives value (i % 4) of the chunks named by lanes
// i / 4, 4 + i / 4, 8 + i / 4 and 12 + i / 4 -- four rows at one column, the MFMA k order.
__device__ __forceinline__ i16x4 lds_tr_read(const char *lds_addr) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)(lds_addr));
}

// BR = 16: operands of v_mfma_f32_16x16x32: lane l holds row/col l % 16, k slots 8 * (l / 16) + 0..7.
//          The product is taken as (X^T tile) x (W^T fragment) so that a lane ends up with 4
//          consecutive columns n of one output row (16-byte stores).
// BR = 32: v_mfma_f32_32x32x16: lane l holds row/col l % 32, k slots 8 * (l / 32) + 0..7; weights
//          are the first operand, so a lane holds one column n and 16 rows.
template <bool BF16, int BR, int NT, int SPW>
__global__ void __launch_bounds__(256) bcr_spmm_mma(MmaParams p) {
    constexpr int NSUB = BR == 16 ? 16 : 32;
    constexpr int TN = NT * NSUB;
    constexpr int KS = BR == 16 ? 32 : 16;
    constexpr int ROWB = TN * 2 + 32;            // LDS row pitch in bytes
    constexpr int SLOTS = TN / 8;                // 16-byte slots per staged row
    constexpr int PF = kMmaMaxChunkRows * SLOTS / 256;
    constexpr int G = 4 * SPW;                   // strips per workgroup
    using Acc = typename std::conditional<BR == 16, f32x4, f32x16>::type;

    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int stage_bytes = (p.chunk_rows + 1) * ROWB;

    // workgroup -> (tile, strip group); all groups of a tile run on the same XCD
    // (workgroups are dealt to the 8 XCDs round-robin by linear id)
    const int id = blockIdx.x;
    const int xcd = id & 7, slot = id >> 3;
    const int tile = (slot / p.ngroups) * 8 + xcd;
    const int group = slot % p.ngroups;
    if (tile >= p.ntiles) return;
    const int64_t n0 = (int64_t)tile * TN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // zero rows (gather target of padded k slots) of both stages
    if (tid < 2 * (ROWB / 4)) {
        int st = tid / (ROWB / 4), w = tid % (ROWB / 4);
        *reinterpret_cast<unsigned int *>(lds + st * stage_bytes + p.chunk_rows * ROWB + w * 4) = 0u;
    }

    Acc acc[SPW][NT];
#pragma unroll
    for (int s = 0; s < SPW; ++s)
#pragma unroll
        for (int q = 0; q < NT; ++q)
#pragma unroll
            for (int e = 0; e < (BR == 16 ? 4 : 16); ++e) acc[s][q][e] = 0.f;

    // ---- staging of X: global -> registers -> LDS ----
    u32x4 pre[PF];
    auto fetch = [&](int chunk) {
        const int64_t k0 = (int64_t)chunk * p.chunk_rows;
        const int rows = (int)((p.K - k0) < p.chunk_rows ? (p.K - k0) : p.chunk_rows);
#pragma unroll
        for (int i = 0; i < PF; ++i) {
            const int sl = tid + i * 256;
            const int r = sl / SLOTS, cs = sl % SLOTS;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (r < rows) {
                const int64_t n = n0 + cs * 8;
                const unsigned short *src = p.X + (k0 + r) * p.ldx + n;
                if (p.xvec == 8 && n + 8 <= p.N) {
                    v = *reinterpret_cast<const u32x4 *>(src);
                } else if (p.xvec >= 4 && n + 8 <= p.N) {
                    const uint2 a = *reinterpret_cast<const uint2 *>(src);
                    const uint2 b = *reinterpret_cast<const uint2 *>(src + 4);
                    v = u32x4{a.x, a.y, b.x, b.y};
                } else {
                    unsigned int w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (n + e < p.N) w[e >> 1] |= (unsigned int)src[e] << ((e & 1) * 16);
                    v = u32x4{w[0], w[1], w[2], w[3]};
                }
            }
            pre[i] = v;
        }
    };
    auto stash = [&](int stage) {
        char *dst = lds + stage * stage_bytes;
#pragma unroll
        for (int i = 0; i < PF; ++i) {
            const int sl = tid + i * 256;
            const int r = sl / SLOTS, cs = sl % SLOTS;
            if (r < p.chunk_rows) *reinterpret_cast<u32x4 *>(dst + r * ROWB + cs * 16) = pre[i];
        }
    };

    // per-lane constants of the gather
    const int i16 = lane & 15;
    const int kslot = (BR == 16 ? 8 * (lane >> 4) : 8 * (lane >> 5)) + (i16 >> 2);
    const int ncol = (BR == 16 ? 0 : 16 * ((lane >> 4) & 1)) + 4 * (i16 & 3);

    fetch(0);
    stash(0);
    __syncthreads();

    for (int ch = 0; ch < p.nchunks; ++ch) {
        if (ch + 1 < p.nchunks) fetch(ch + 1);
        const char *stage = lds + (ch & 1) * stage_bytes + ncol * 2;
#pragma unroll
        for (int s = 0; s < SPW; ++s) {
            const int t = group * G + s * 4 + wave;       // stored strip of this wave
            if (t >= p.nbr) continue;
            const int32_t *kp = p.kstep_ptr + (int64_t)t * (p.nchunks + 1) + ch;
            const int ks0 = kp[0], ks1 = kp[1];
            for (int ks = ks0; ks < ks1; ++ks) {
                const i16x8 w = *reinterpret_cast<const i16x8 *>(p.afrag + (int64_t)ks * 512 + lane * 8);
                const int r0 = p.kidx[(int64_t)ks * KS + kslot];
                const int r1 = p.kidx[(int64_t)ks * KS + kslot + 4];
                const char *a0 = stage + r0 * ROWB;
                const char *a1 = stage + r1 * ROWB;
#pragma unroll
                for (int q = 0; q < NT; ++q) {
                    const i16x4 lo = lds_tr_read(a0 + q * NSUB * 2);
                    const i16x4 hi = lds_tr_read(a1 + q * NSUB * 2);
                    const i16x8 x = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    if constexpr (BR == 16) acc[s][q] = mfma16<BF16>(x, w, acc[s][q]);
                    else acc[s][q] = mfma32<BF16>(w, x, acc[s][q]);
                }
            }
        }
        if (ch + 1 < p.nchunks) stash((ch + 1) & 1);
        __syncthreads();
    }

    // ---- write the strip tiles of Y (original row order) ----
#pragma unroll
    for (int s = 0; s < SPW; ++s) {
        const int t = group * G + s * 4 + wave;
        if (t >= p.nbr) continue;
        const int64_t row0 = (int64_t)p.strip_order[t] * BR;
#pragma unroll
        for (int q = 0; q < NT; ++q) {
            if constexpr (BR == 16) {
                // D[n][m]: lane holds m = lane % 16, n = 4 * (lane / 16) + 0..3
                const int64_t n = n0 + q * 16 + 4 * (lane >> 4);
                float *dst = p.Y + (row0 + (lane & 15)) * p.ldy + n;
                if (p.yvec == 4 && n + 4 <= p.N) {
                    *reinterpret_cast<f32x4 *>(dst) = acc[s][q];
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (n + e < p.N) dst[e] = acc[s][q][e];
                }
            } else {
                // D[m][n]: lane holds n = lane % 32, m = 8 * (e / 4) + 4 * (lane / 32) + e % 4
                const int64_t n = n0 + q * 32 + (lane & 31);
                if (n < p.N) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int m = 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                        p.Y[(row0 + m) * p.ldy + n] = acc[s][q][e];
                    }
                }
            }
        }
    }
}

bool mma_supported(const grim_bcr_matrix *A) { return A->mma.present; }

template <bool BF16, int BR, int NT, int SPW>
static grim_status launch_mma_inst(const MmaParams &p, hipStream_t stream) {
    constexpr int TN = NT * (BR == 16 ? 16 : 32);
    constexpr int ROWB = TN * 2 + 32;
    const size_t lds = 2 * (size_t)(p.chunk_rows + 1) * ROWB;
    const int64_t tiles8 = ((int64_t)p.ntiles + 7) / 8 * 8;
    const int64_t nwg = tiles8 * p.ngroups;
    if (nwg > 0x7fffffff) return GRIM_ERR_SHAPE;
    auto kern = bcr_spmm_mma<BF16, BR, NT, SPW>;
    if (lds > 64 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
            (void)hipGetLastError();
            return GRIM_ERR_DEVICE;
        }
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(256), lds, stream, p);
    return hipGetLastError() == hipSuccess ? GRIM_OK : GRIM_ERR_DEVICE;
}

template <bool BF16, int BR>
static grim_status launch_mma_br(MmaParams &p, int tile_n, int spw, hipStream_t stream) {
    constexpr int NSUB = BR == 16 ? 16 : 32;
    const int nt = tile_n / NSUB;
    p.ntiles = (int32_t)((p.N + tile_n - 1) / tile_n);
    p.ngroups = (p.nbr + 4 * spw - 1) / (4 * spw);
#define GRIM_CASE(NT_, SPW_) \
    if (nt == NT_ && spw == SPW_) return launch_mma_inst<BF16, BR, NT_, SPW_>(p, stream);
    if constexpr (BR == 16) {
        GRIM_CASE(2, 1) GRIM_CASE(2, 2) GRIM_CASE(2, 4)
        GRIM_CASE(4, 1) GRIM_CASE(4, 2) GRIM_CASE(4, 4)
        GRIM_CASE(8, 1) GRIM_CASE(8, 2)
    } else {
        GRIM_CASE(1, 1) GRIM_CASE(1, 2) GRIM_CASE(1, 4)
        GRIM_CASE(2, 1) GRIM_CASE(2, 2) GRIM_CASE(2, 4)
        GRIM_CASE(4, 1) GRIM_CASE(4, 2)
    }
#undef GRIM_CASE
    return GRIM_ERR_UNSUPPORTED;
}

grim_status launch_spmm_mma(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, float *Y, int64_t ldy,
                            int32_t tile_n, int32_t strips_per_wg, hipStream_t stream) {
    if (!A->mma.present) return GRIM_ERR_UNSUPPORTED;
    if (tile_n != 0 && tile_n != 32 && tile_n != 64 && tile_n != 128) return GRIM_ERR_UNSUPPORTED;
    if (strips_per_wg != 0 && strips_per_wg != 4 && strips_per_wg != 8 && strips_per_wg != 16) return GRIM_ERR_UNSUPPORTED;
    const int tn = tile_n ? tile_n : (N <= 32 ? 32 : 64);
    int spw;
    if (strips_per_wg) {
        spw = strips_per_wg / 4;
    } else {
        // Every strip group of a tile re-reads the tile's rows of X (through L2), so take the
        // largest group that still leaves about one workgroup per compute unit.
        const int64_t tiles = (N + tn - 1) / tn;
        spw = A->nbr > 8 ? 4 : A->nbr > 4 ? 2 : 1;
        while (spw > 1 && tiles * ((A->nbr + 4 * spw - 1) / (4 * spw)) < 256) spw >>= 1;
    }
    if (tn == 128 && spw > 2) spw = 2;   // accumulator registers
    MmaParams p;
    p.afrag = A->mma.d_afrag;
    p.kidx = A->mma.d_kidx;
    p.kstep_ptr = A->mma.d_kstep_ptr;
    p.strip_order = A->dev.strip_order;
    p.X = static_cast<const unsigned short *>(X);
    p.Y = Y;
    p.N = N; p.ldx = ldx; p.ldy = ldy;
    p.K = (int32_t)A->K; p.nbr = (int32_t)A->nbr; p.nchunks = A->mma.nchunks; p.chunk_rows = A->mma.chunk_rows;
    const uintptr_t xa = reinterpret_cast<uintptr_t>(X), ya = reinterpret_cast<uintptr_t>(Y);
    p.xvec = (xa % 16 == 0 && ldx % 8 == 0) ? 8 : (xa % 8 == 0 && ldx % 4 == 0) ? 4 : 1;
    p.yvec = (ya % 16 == 0 && ldy % 4 == 0) ? 4 : 1;
    const bool bf = A->dtype == GRIM_BF16;
    if (A->BR == 16) return bf ? launch_mma_br<true, 16>(p, tn, spw, stream) : launch_mma_br<false, 16>(p, tn, spw, stream);
    return bf ? launch_mma_br<true, 32>(p, tn, spw, stream) : launch_mma_br<false, 32>(p, tn, spw, stream);
}

}  // namespace grim

// Portable SpMM kernel on the vector ALUs for Y = W_bcr * X (Section 3.1: CONV as GEMM on the im2col matrix).
// Any element type, BR <= 64.  A workgroup of 4 to 16 waves owns one row strip x 64 columns of X; each wave walks its
// share of the strip's blocks in ascending column-block order and the waves' sums are added in a fixed order;
// every gathered X value is loaded once and reused by all kept rows of the block
// (the load-redundancy elimination of Section 4.4, here a consequence of treating the block as a small dense
// matrix).
#include "spmm_common.hpp"

namespace grim {

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

// Waves of a workgroup: they share a strip's column blocks.  A block costs a wave three dependent fetches (block
// header, column indices, values of X), so the more waves the shorter the chain: as many as their sums leave room
// for in 64 KB of LDS (256 x 256 in 16 x 16 blocks, 64 columns: 57 us with one wave per strip, 18 us with 4).
constexpr int fma_waves(int brcap) { return brcap <= 16 ? 16 : brcap <= 32 ? 8 : 4; }
constexpr int kFmaBatch = 8;     // gathered values of X in flight per lane

template <int DT, int BRCAP>
__global__ void __launch_bounds__(fma_waves(BRCAP) * 64) bcr_spmm_fma(FmaParams p) {
    using T = typename Elem<DT>::type;
    constexpr int kFmaWaves = fma_waves(BRCAP);
    __shared__ float part[kFmaWaves * BRCAP * 64];       // [wave][strip row][column]: 64 KB
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t t = blockIdx.x;                        // stored strip
    const int64_t n = (int64_t)blockIdx.y * 64 + lane;
    const bool live = n < p.N;
    const int64_t nc = live ? n : p.N - 1;               // idle lanes re-read the last column
    const T *X = static_cast<const T *>(p.X);
    const T *W = static_cast<const T *>(p.weights);
    float *mine = part + (wave * BRCAP) * 64 + lane;     // this lane's column of the wave's sums, one entry per strip row
#pragma unroll
    for (int r = 0; r < BRCAP; ++r) mine[r * 64] = 0.f;
    // Wave w takes the column blocks w, w + waves, ... in ascending order.  A block's sums are formed per KEPT row
    // (rank i = 0 .. kept - 1), in groups of four ranks without a test of the row mask inside (a test per row and
    // column made the loop a chain of 128 branches); rank i is then added to the entry of the row it stands for.
    // Within a block the gathered values of X are fetched kFmaBatch at a time, all loads of a batch issued before the
    // first is used.
    for (int64_t c = wave; c < p.nbc; c += kFmaWaves) {
        const int64_t b = t * p.nbc + c;
        const uint64_t mask = p.rowmask[b];
        const int32_t cp0 = p.col_ptr[b];
        const int32_t kc = p.col_ptr[b + 1] - cp0;
        if (mask == 0 || kc == 0) continue;
        const T *wb = W + p.blk_ptr[b];
        const int32_t nk = __builtin_popcountll(mask);
        // A block of at most 256 kept weights is fetched once, element e by lane e % 64 (four loads, all in flight with
        // the block's column indices), and a weight is then read out of its lane's register.
        const int32_t nel = nk * kc;
        const bool in_lanes = BRCAP <= 16 && nel <= 4 * 64;
        float wl[4] = {0.f, 0.f, 0.f, 0.f};
        if (in_lanes) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int32_t e = q * 64 + lane < nel ? q * 64 + lane : nel - 1;
                wl[q] = to_f32<DT>(wb[e]);
            }
        }
        // MODE 0: weights from memory, 1: out of the lanes of wl[0] (at most 64 of them), 2: out of wl[0..3]
        auto weight = [&](auto mode, int32_t e) {       // e: the same for the whole wave
            constexpr int MODE = decltype(mode)::value;
            if constexpr (MODE == 0) {
                return to_f32<DT>(wb[e]);
            } else {
                const int32_t q = e >> 6;
                const float v = MODE == 1 ? wl[0] : q == 0 ? wl[0] : q == 1 ? wl[1] : q == 2 ? wl[2] : wl[3];
                return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), e & 63));
            }
        };
        float acc[BRCAP];
#pragma unroll
        for (int i = 0; i < BRCAP; ++i) acc[i] = 0.f;
        auto columns = [&](auto mode) {
            for (int32_t j0 = 0; j0 < kc; j0 += kFmaBatch) {
                float xv[kFmaBatch];
#pragma unroll
                for (int u = 0; u < kFmaBatch; ++u) {
                    const int32_t j = j0 + u < kc ? j0 + u : kc - 1;
                    const int64_t k = c * p.BC + p.col_idx[cp0 + j];
                    xv[u] = to_f32<DT>(X[k * p.ldx + nc]);
                }
#pragma unroll
                for (int u = 0; u < kFmaBatch; ++u) {
                    if (j0 + u < kc) {
#pragma unroll
                        for (int i4 = 0; i4 < BRCAP; i4 += 4) {
                            if (i4 < nk) {              // (ranks past the last kept row re-use its weights; never stored)
#pragma unroll
                                for (int i = i4; i < i4 + 4; ++i) {
                                    const int32_t ic = i < nk ? i : nk - 1;
                                    acc[i] = __builtin_fmaf(weight(mode, ic * kc + j0 + u), xv[u], acc[i]);
                                }
                            }
                        }
                    }
                }
            }
        };
        if (!in_lanes) columns(std::integral_constant<int, 0>{});
        else if (nel <= 64) columns(std::integral_constant<int, 1>{});
        else columns(std::integral_constant<int, 2>{});
        uint64_t m = mask;
#pragma unroll
        for (int i = 0; i < BRCAP; ++i) {
            if (i < nk) {                               // same for the whole wave
                const int r = __builtin_ctzll(m);
                m &= m - 1;
                mine[r * 64] += acc[i];
            }
        }
    }
    __syncthreads();
    // the strip's rows are dealt to the waves; a row's sums are added in wave order
    const int64_t row0 = (int64_t)p.strip_order[t] * p.BR;
    for (int r = wave; r < p.BR; r += kFmaWaves) {
        float s = part[r * 64 + lane];
#pragma unroll
        for (int w = 1; w < kFmaWaves; ++w) s += part[(w * BRCAP + r) * 64 + lane];
        if (live) p.Y[(row0 + r) * p.ldy + n] = s;
    }
}

template <int DT>
static grim_status launch_fma_dt(const FmaParams &p, int32_t BR, int64_t nbr, hipStream_t stream) {
    if ((p.N + 63) / 64 > 65535 || nbr > 0x7fffffff) return GRIM_ERR_SHAPE;
    dim3 grid((unsigned)nbr, (unsigned)((p.N + 63) / 64));
    if (BR <= 16) hipLaunchKernelGGL((bcr_spmm_fma<DT, 16>), grid, dim3(fma_waves(16) * 64), 0, stream, p);
    else if (BR <= 32) hipLaunchKernelGGL((bcr_spmm_fma<DT, 32>), grid, dim3(fma_waves(32) * 64), 0, stream, p);
    else hipLaunchKernelGGL((bcr_spmm_fma<DT, 64>), grid, dim3(fma_waves(64) * 64), 0, stream, p);
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


}  // namespace grim

// SpMM kernels for Y = W_bcr * X (Section 3.1: CONV as GEMM on the im2col matrix).
//
//  * bcr_spmm_fma  -- portable kernel on the vector ALUs.  Any element type, BR <= 64.
//    One wave owns one row strip x 64 columns of X and walks the strip's blocks in
//    ascending column-block order; every gathered X value is loaded once and reused
//    by all kept rows of the block (the load-redundancy elimination of Section 4.4,
//    here a consequence of treating the block as a small dense matrix).
//  * bcr_spmm_mma  -- matrix-core kernel for fp16 / bf16 with BR = 16 or 32.
//    A workgroup owns a tile of TN columns of X and a group of row strips.  Chunks of
//    consecutive X rows are staged in LDS once per workgroup (tiling, Section 4.4) by
//    dedicated producer waves (global -> registers -> LDS), two chunks ahead of the
//    consumer waves.  Each consumer wave gathers the rows its strips keep with LDS
//    transpose reads straight into MFMA operand layout and multiplies them with the
//    kept rows of the blocks' weights (lanes of rows a block does not keep multiply
//    zeros).  Strips are dealt to waves in stored (work-sorted, Section 4.2) order so
//    the waves of a workgroup carry near-equal work.
//    Accumulation is fp32, order fixed, no atomics.
#include <hip/hip_runtime.h>

#include <atomic>

#include <cstdlib>
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
    const unsigned char *recs;
    const int32_t *cptr;
    const int32_t *bptr;
    const int32_t *strip_order;
    const unsigned short *X;
    float *Y;
    int64_t N, ldx, ldy;
    int32_t K, nbr, nchunks, chunk_rows;
    int32_t ntiles, ngroups;
    int32_t amax;   // 16-byte units of records one LDS stage must hold
    int32_t xvec;   // widest aligned vector (elements: 8, 4 or 1) for rows of X
    int32_t yvec;   // 4 when rows of Y allow aligned float4 stores, else 1
#ifdef GRIM_DBG
    long long *dbg;
#endif
};

#ifdef GRIM_DBG
#define GRIM_STAMP(slot, j) do { if (p.dbg && blockIdx.x == 8 && lane == 0) p.dbg[((j) + 1) * 16 + (slot)] = (long long)__builtin_amdgcn_s_memtime(); } while (0)
#else
#define GRIM_STAMP(slot, j) do { } while (0)
#endif

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
__device__ __forceinline__ i16x4 lds_tr_read_at(unsigned int lds_byte_address) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)(uintptr_t)lds_byte_address);
}
__device__ __forceinline__ i16x4 lds_tr_read(const char *lds_addr) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)(lds_addr));
}

// Staged rows have no padding; the 16-byte chunks of a row are XOR-swizzled by the row
// number so that the four rows one transpose read touches fall into different bank groups
// whenever their numbers differ mod 4 (mod 8 for 128-byte rows, where consecutive rows
// already sit in opposite halves of the 256-byte bank line; measured 3-7 % faster).
template <int CPR>   // 16-byte chunks per staged row
__device__ __forceinline__ int swizzle(int row) {
    return CPR == 8 ? (((row >> 1) & 3) << 1) : CPR > 8 ? ((row & 3) << 1) : (((row >> 1) & 1) << 1);
}

// LDS bytes of one stage: staged X rows + zero row, then room for amax 16-byte units of
// records rounded up to whole 1 KB slots
__host__ __device__ inline int mma_stage_bytes(int chunk_rows, int pitch, int amax) {
    return (chunk_rows + 1) * pitch + ((amax * 16 + 1023) / 1024 + 1) * 1024;
}

// Workgroup = NW consumer waves + NP producer waves; LDS holds two stages, each
//   [chunk_rows staged rows of X | one zero row | the chunk's step records].
// Everything a chunk needs -- the X rows of the tile and the record regions of the group's strips,
// one contiguous byte range -- is cut into 1 KB slots (one 16-byte load per lane).  The producers
// form two teams that alternate chunks; the NM members of a team share a chunk's slots.  A team
// issues the loads of chunk c + 2 into registers while the consumers multiply chunk c, and
// writes them to the free stage one chunk later, so two chunks are in flight per workgroup and
// global load latency spans two chunk periods.  One barrier per chunk, no atomics.
//
// BR = 16: operands of v_mfma_f32_16x16x32: lane l holds row/col l % 16, k slots 8 * (l / 16) + 0..7.
//          The product is taken as (X^T tile) x (W^T fragment) so that a lane ends up with 4
//          consecutive columns n of one output row (16-byte stores).
// BR = 32: v_mfma_f32_32x32x16: lane l holds row/col l % 32, k slots 8 * (l / 32) + 0..7; weights
//          are the first operand, so a lane holds one column n and 16 rows.
template <bool BF16, int BR, int NT, int SPW, int NW, int NP, int SX, int SR>
__global__ void __launch_bounds__((NW + NP) * 64) bcr_spmm_mma(MmaParams p) {
    constexpr int NSUB = BR == 16 ? 16 : 32;
    constexpr int TN = NT * NSUB;
    constexpr int PITCH = TN * 2;                // LDS row pitch in bytes (no padding)
    constexpr int CPR = PITCH / 16;              // 16-byte chunks per staged row
    constexpr int RPS = 1024 / PITCH;            // staged rows per slot
    constexpr int G = NW * SPW;                  // strips per workgroup
    constexpr int NM = NP / 2;                   // members of a producer team
    using Acc = typename std::conditional<BR == 16, f32x4, f32x16>::type;

    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int xbytes = (p.chunk_rows + 1) * PITCH;            // X rows + zero row
    const int stage_bytes = mma_stage_bytes(p.chunk_rows, PITCH, p.amax);
    constexpr int KS = BR == 16 ? 32 : 16;       // k slots per step
    constexpr int HDR = KS * 2 + (KS / 8) * 8;   // header bytes per step
    // after the two stages: (first step, region start in 16-byte units) of (chunk, strip of this
    // group), [nchunks][G + 1]
    const int2 *tab = reinterpret_cast<const int2 *>(lds + 2 * stage_bytes);

    // workgroup -> (tile, strip group); all groups of a tile run on the same XCD
    // (workgroups are dealt to the 8 XCDs round-robin by linear id)
    const int id = blockIdx.x;
    const int xcd = id & 7, slot = id >> 3;
    const int tile = (slot / p.ngroups) * 8 + xcd;
    const int group = slot % p.ngroups;
    if (tile >= p.ntiles) return;
    // A ragged last tile is shifted left to end exactly at N when that keeps its rows 8-byte
    // aligned: it then overlaps its neighbour and both write the same bits to the shared columns
    // (a column's sum does not depend on the tile that computes it), and no lane has to stage a
    // partial 16-byte piece element by element.
    int64_t n0 = (int64_t)tile * TN;
    if (n0 + TN > p.N && p.N >= TN && ((p.N - TN) & 3) == 0) n0 = p.N - TN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int t0 = group * G;                                  // first stored strip of the group
    const int t1 = t0 + G < p.nbr ? t0 + G : p.nbr;

    // zero rows (gather target of padded k slots), one per stage
    if (tid < 2 * (PITCH / 4)) {
        const int st = tid / (PITCH / 4), w = tid % (PITCH / 4);
        *reinterpret_cast<unsigned int *>(lds + st * stage_bytes + p.chunk_rows * PITCH + w * 4) = 0u;
    }

    if (wave >= NW) {
        // ---- producers ----
        const int q = wave - NW, team = q & 1, mem = q >> 1;
        // this lane's place in an X slot: row (within the slot's RPS rows) and 16-byte chunk
        const int lrow = lane / CPR;
        const int c = (lane % CPR) ^ swizzle<CPR>(lrow);      // slots are RPS rows apart: same swizzle
        const int64_t n = n0 + c * 8;
        // Lanes whose 8 columns lie inside the row take the pipelined path when the rows of X are
        // at least 8-byte aligned: plain 16-byte (or two 8-byte) loads into registers, no test or
        // merge after a load, so all loads of a chunk are in flight together.  Lanes straddling the
        // end of the row (N not a multiple of 8) or unaligned rows are staged element-wise when the
        // chunk is written; lanes past the end of the row stage nothing (their columns are never
        // stored).
        const bool full = p.xvec >= 4 && n + 8 <= p.N;
        const bool part = !full && n < p.N;
        const bool wide = p.xvec == 8 && (n0 & 7) == 0;
        // interior tile of 16-byte-aligned X: every lane is full, no per-lane control flow at all
        const bool all_wide = wide && n0 + TN <= p.N;
        u32x4 RX[SX], RR[SR];

        struct Shape { int xs, nrs, rows; int64_t k0, rbyte; };
        // chunks 0 and 1 are shaped from global memory (the table is not filled yet), later
        // chunks from the LDS table
        auto shape_of = [&](int chunk, bool from_table) {
            Shape h;
            int b0, units;
            if (from_table) {
                b0 = tab[chunk * (G + 1)].y;
                units = tab[chunk * (G + 1) + G].y - b0;
            } else {
                const int32_t *bp = p.bptr + (int64_t)chunk * (p.nbr + 1);
                b0 = bp[t0];
                units = bp[t1] - b0;
            }
            h.rbyte = (int64_t)b0 * 16;
            h.nrs = (units * 16 + 1023) >> 10;
            h.k0 = (int64_t)chunk * p.chunk_rows;
            h.rows = (int)((p.K - h.k0) < p.chunk_rows ? (p.K - h.k0) : p.chunk_rows);
            h.xs = (h.rows + RPS - 1) / RPS;
            return h;
        };
        auto load_chunk = [&](int chunk, bool from_table) {
            const Shape h = shape_of(chunk, from_table);
            const char *rsrc = reinterpret_cast<const char *>(p.recs) + h.rbyte + lane * 16;
#pragma unroll
            for (int i = 0; i < SR; ++i) {
                const int sl = mem + i * NM;
                if (sl < h.nrs) RR[i] = *reinterpret_cast<const u32x4 *>(rsrc + (int64_t)sl * 1024);
            }
            if (all_wide) {
                const unsigned short *xsrc = p.X + h.k0 * p.ldx + n;
#pragma unroll
                for (int i = 0; i < SX; ++i) {
                    int row = (mem + i * NM) * RPS + lrow;
                    row = row < h.rows ? row : h.rows - 1;
                    RX[i] = *reinterpret_cast<const u32x4 *>(xsrc + (int64_t)row * p.ldx);
                }
            } else if (full) {
                // rows past the end of the chunk are clamped to its last row (never stored / read)
                const unsigned short *xsrc = p.X + h.k0 * p.ldx + n;
                if (wide) {
#pragma unroll
                    for (int i = 0; i < SX; ++i) {
                        int row = (mem + i * NM) * RPS + lrow;
                        row = row < h.rows ? row : h.rows - 1;
                        RX[i] = *reinterpret_cast<const u32x4 *>(xsrc + (int64_t)row * p.ldx);
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < SX; ++i) {
                        int row = (mem + i * NM) * RPS + lrow;
                        row = row < h.rows ? row : h.rows - 1;
                        const unsigned short *g = xsrc + (int64_t)row * p.ldx;
                        const uint2 a = *reinterpret_cast<const uint2 *>(g);
                        const uint2 b = *reinterpret_cast<const uint2 *>(g + 4);
                        RX[i].x = a.x; RX[i].y = a.y; RX[i].z = b.x; RX[i].w = b.y;
                    }
                }
            }
        };
        auto store_chunk = [&](int chunk, bool from_table) {
            const Shape h = shape_of(chunk, from_table);
            char *sbase = lds + (chunk & 1) * stage_bytes;
#pragma unroll
            for (int i = 0; i < SR; ++i) {
                const int sl = mem + i * NM;
                if (sl < h.nrs) *reinterpret_cast<u32x4 *>(sbase + xbytes + sl * 1024 + lane * 16) = RR[i];
            }
            if (all_wide) {
#pragma unroll
                for (int i = 0; i < SX; ++i) {
                    const int sl = mem + i * NM;
                    if (sl * RPS + lrow < h.rows) *reinterpret_cast<u32x4 *>(sbase + sl * 1024 + lane * 16) = RX[i];
                }
            } else if (full) {
#pragma unroll
                for (int i = 0; i < SX; ++i) {
                    const int sl = mem + i * NM;
                    if (sl * RPS + lrow < h.rows) *reinterpret_cast<u32x4 *>(sbase + sl * 1024 + lane * 16) = RX[i];
                }
            }
            if (!all_wide && part) {
                for (int sl = mem; sl < h.xs; sl += NM) {
                    const int row = sl * RPS + lrow;
                    if (row < h.rows) {
                        const unsigned short *g = p.X + (h.k0 + row) * p.ldx + n;
                        unsigned int w[4] = {0u, 0u, 0u, 0u};
                        for (int e = 0; e < 8; ++e)
                            if (n + e < p.N) w[e >> 1] |= (unsigned int)g[e] << ((e & 1) * 16);
                        *reinterpret_cast<u32x4 *>(sbase + sl * 1024 + lane * 16) = u32x4{w[0], w[1], w[2], w[3]};
                    }
                }
            }
        };

        if (q < 3) GRIM_STAMP(q * 4 + 0, -1);
        if (team < p.nchunks) load_chunk(team, false);        // team 0: chunk 0, team 1: chunk 1
        if (q < 3) GRIM_STAMP(q * 4 + 1, -1);
        if (team == 0) store_chunk(0, false);
        if (q < 3) GRIM_STAMP(q * 4 + 2, -1);
        __syncthreads();
        for (int j = 0; j < p.nchunks; ++j) {
            if (q < 3) GRIM_STAMP(q * 4 + 0, j);
            if ((j & 1) == team) {
                if (j + 2 < p.nchunks) load_chunk(j + 2, true);   // registers were emptied one chunk ago
            } else {
                if (j + 1 < p.nchunks) store_chunk(j + 1, true);  // stage (j + 1) % 2 was read last in chunk j - 1
            }
            if (q < 3) GRIM_STAMP(q * 4 + 2, j);
            __syncthreads();
            if (q < 3) GRIM_STAMP(q * 4 + 3, j);
        }
        return;
    }

    // ---- consumers ----
    Acc acc[SPW][NT];
#pragma unroll
    for (int s = 0; s < SPW; ++s)
#pragma unroll
        for (int q = 0; q < NT; ++q)
#pragma unroll
            for (int e = 0; e < (BR == 16 ? 4 : 16); ++e) acc[s][q][e] = 0.f;

    // per-lane constants of the gather: byte column inside a sub-tile
    const int i16 = lane & 15;
    const int ncolb = ((BR == 16 ? 0 : 16 * ((lane >> 4) & 1)) + 4 * (i16 & 3)) * 2;
    const int cl = ncolb >> 4, within = ncolb & 15;

    int tstrip[SPW];
#pragma unroll
    for (int s = 0; s < SPW; ++s) tstrip[s] = t0 + s * NW + wave;   // stored strips of this wave

    // fill the table while the producers fetch the first chunk (strips past the last one get
    // the chunk's end, i.e. an empty range)
    {
        int2 *wtab = reinterpret_cast<int2 *>(lds + 2 * stage_bytes);
        for (int e = tid; e < p.nchunks * (G + 1); e += NW * 64) {
            const int ch = e / (G + 1), i = e % (G + 1);
            const int t = t0 + i < p.nbr ? t0 + i : p.nbr;
            wtab[e] = int2{p.cptr[(int64_t)ch * (p.nbr + 1) + t], p.bptr[(int64_t)ch * (p.nbr + 1) + t]};
        }
    }
    // per-lane constants of the weight fragment: output row inside the strip and k group
    const int m_row = BR == 16 ? (lane & 15) : (lane & 31);
    const int kgroup = BR == 16 ? (lane >> 4) : (lane >> 5);
    const unsigned int below = (1u << m_row) - 1u;
    const int hdr_rows = (kgroup * 4 + (i16 >> 2)) * 4;        // this lane's pair of staged-row numbers
    const int hdr_desc = KS * 2 + kgroup * 8;                  // its group's (row mask, payload offset)

    // A step's header holds the staged-row numbers of its k slots and, per group of 8 slots, the
    // block's row mask and the place of its weights; the weights of a lane (its row of the
    // group's block if the block keeps that row, else zeros) can only be read once the header
    // is there.  Steps are therefore taken two at a time, with the headers of the next pair
    // requested before the current pair is multiplied: per pair one LDS round trip for the
    // weights and X values of both steps instead of two dependent ones per step.
    struct Hdr { unsigned int rr; uint2 dsc; };
    auto load_hdr = [&](const char *region, int r) {
        Hdr f;
        const char *h = region + r * HDR;
        f.rr = *reinterpret_cast<const unsigned int *>(h + hdr_rows);
        f.dsc = *reinterpret_cast<const uint2 *>(h + hdr_desc);
        return f;
    };
    auto load_w = [&](const char *region, const Hdr &f) {
        const bool kept = (f.dsc.x >> m_row) & 1u;
        const int idx = kept ? __builtin_popcount(f.dsc.x & below) : 0;
        const i16x8 w = *reinterpret_cast<const i16x8 *>(region + (f.dsc.y + idx) * 16);
        return kept ? w : i16x8{0, 0, 0, 0, 0, 0, 0, 0};
    };
    auto load_x = [&](const char *stage, const Hdr &f, i16x8 (&x)[NT]) {
        const int r0 = f.rr & 0xffff, r1 = f.rr >> 16;
        const int sw0 = swizzle<CPR>(r0), sw1 = swizzle<CPR>(r1);
        const char *x0 = stage + r0 * PITCH + within;
        const char *x1 = stage + r1 * PITCH + within;
#pragma unroll
        for (int q = 0; q < NT; ++q) {
            const int cq = q * (NSUB / 8) + cl;
            const i16x4 lo = lds_tr_read(x0 + ((cq ^ sw0) << 4));
            const i16x4 hi = lds_tr_read(x1 + ((cq ^ sw1) << 4));
            x[q] = i16x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        }
    };

    __syncthreads();
    // (number of steps, region offset) of this wave's strips in a chunk, read one chunk ahead so
    // that the look-up is off the critical path after the barrier
    struct Entry { int nst, off; };
    auto entries_of = [&](int ch, Entry (&en)[SPW]) {
        const int2 *row = tab + ch * (G + 1);
        const int2 base = row[0];
#pragma unroll
        for (int s = 0; s < SPW; ++s) {
            const int2 e0 = row[s * NW + wave], e1 = row[s * NW + wave + 1];
            en[s].nst = e1.x - e0.x;
            en[s].off = (e0.y - base.y) * 16;
        }
    };
    Entry en[SPW], en_next[SPW];
    entries_of(0, en);
    for (int ch = 0; ch < p.nchunks; ++ch) {
        const char *stage = lds + (ch & 1) * stage_bytes;
        const char *frs = stage + xbytes;
        if (wave == 0) GRIM_STAMP(12, ch);
        entries_of(ch + 1 < p.nchunks ? ch + 1 : ch, en_next);
#pragma unroll
        for (int s = 0; s < SPW; ++s) {
            const int nst = en[s].nst;
            if (nst <= 0) continue;
            const char *region = frs + en[s].off;
            Hdr ha = load_hdr(region, 0), hb = load_hdr(region, nst > 1 ? 1 : 0);
            for (int r = 0; r < nst; r += 2) {
                const i16x8 wa = load_w(region, ha), wb = load_w(region, hb);
                i16x8 xa[NT], xb[NT];
                load_x(stage, ha, xa);
                load_x(stage, hb, xb);
                const int ra = r + 2 < nst ? r + 2 : nst - 1, rb = r + 3 < nst ? r + 3 : nst - 1;
                ha = load_hdr(region, ra);
                hb = load_hdr(region, rb);
#pragma unroll
                for (int q = 0; q < NT; ++q) {
                    if constexpr (BR == 16) acc[s][q] = mfma16<BF16>(xa[q], wa, acc[s][q]);
                    else acc[s][q] = mfma32<BF16>(wa, xa[q], acc[s][q]);
                }
                if (r + 1 < nst) {
#pragma unroll
                    for (int q = 0; q < NT; ++q) {
                        if constexpr (BR == 16) acc[s][q] = mfma16<BF16>(xb[q], wb, acc[s][q]);
                        else acc[s][q] = mfma32<BF16>(wb, xb[q], acc[s][q]);
                    }
                }
            }
        }
        if (wave == 0) GRIM_STAMP(13, ch);
#pragma unroll
        for (int s = 0; s < SPW; ++s) en[s] = en_next[s];
        __syncthreads();
        if (wave == 0) GRIM_STAMP(14, ch);
    }
    if (wave == 0) GRIM_STAMP(15, p.nchunks);

    // ---- write the strip tiles of Y (original row order) ----
#pragma unroll
    for (int s = 0; s < SPW; ++s) {
        const int t = tstrip[s];
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

// ------------------------------------------------------------------------------------------
// row-gathering matrix-core kernel (fp16 / bf16; block heights that divide 16 or are multiples of
// 16: the rows of the matrix in stored order are cut into runs of 16, "strips" below)
//
// Workgroup = (tile of 64 columns of X, one 16-row strip); its 4 waves split the strip's steps
// (i.e. K) between them and add their partial tiles in a fixed order at the end -- the only
// barrier.  A wave works on its own: it reads the row numbers and block descriptors of a batch
// of steps, then fetches exactly the rows of X those steps multiply (8 lanes per 128-byte row
// piece) and the kept rows of the blocks' weights straight into registers, parks the X rows of
// one step in a private 4 KB LDS buffer in k-slot order, and reads them back with transpose
// reads as MFMA operands.  No producer/consumer hand-over: latency is covered by the four
// workgroups a compute unit holds and by the batch of loads a wave has in flight.
// Unlike the staged kernel a row of X is fetched once per strip that keeps it (not once per
// group of strips), but only kept rows are fetched, and every compute unit has work even when
// the tiles are few.
// ------------------------------------------------------------------------------------------
// Waves that split a long strip's steps in the few-workgroups form (template flag EIGHT).  A 36-step strip of a 14 x 14
// layer: 8 waves of the row-gathering kernel (4 steps per batch) 7.66 us, 12 waves 7.63, 16 waves 8.56; the convolution
// kernel (3 steps per batch) 11.0 us with 8, 8.6 us with 12 -- every wave then needs one batch only --, 9.7 us with 16.
constexpr int kGatherLongWaves = 8, kConvLongWaves = 12;
static_assert(kConvLongWaves == 12, "the launcher names the instantiations");

// Workgroup id -> (tile of columns, unit of the tile's work) for the kernels whose workgroups of one
// tile fetch the same rows: ids are dealt to the 8 XCDs round-robin, each XCD has its own L2, so a
// tile's units go to one XCD.  With that alone the last ntiles % 8 tiles (all of them when there
// are fewer than 8: one tile for N <= 64) would leave XCDs idle, so each of those tiles is cut into
// 2^shift interleaved parts, enough for a multiple of 8, and the parts are dealt instead.
struct XcdMap {
    int32_t per_tile;         // units per tile
    int32_t tail_slot0;       // first slot (id / 8) of the tail tiles
    int32_t tail_tile0;       // first tail tile, a multiple of 8
    int32_t shift;            // tail tiles are cut into 1 << shift parts ...
    int32_t per_part;         // ... of this many units
};
static XcdMap xcd_map(int32_t ntiles, int64_t per_tile, int64_t *nwg) {
    XcdMap m;
    const int32_t full = ntiles / 8, r = ntiles % 8;
    m.per_tile = (int32_t)per_tile;
    m.tail_slot0 = (int32_t)(full * per_tile);
    m.tail_tile0 = full * 8;
    m.shift = r == 0 ? 0 : r % 4 == 0 ? 1 : r % 2 == 0 ? 2 : 3;
    m.per_part = (int32_t)((per_tile + (1 << m.shift) - 1) >> m.shift);
    *nwg = 8 * (full * per_tile + (int64_t)((r << m.shift) / 8) * m.per_part);
    return m;
}
// false: the workgroup has no tile
__device__ __forceinline__ bool xcd_map_at(const XcdMap &m, int id, int ntiles, int *tile, int *unit) {
    const int xcd = id & 7, slot = id >> 3;
    if (slot < m.tail_slot0) {
        *tile = (slot / m.per_tile) * 8 + xcd;
        *unit = slot % m.per_tile;
        return true;
    }
    const int s2 = slot - m.tail_slot0;
    const int part = (s2 / m.per_part) * 8 + xcd;
    *tile = m.tail_tile0 + (part >> m.shift);
    *unit = ((s2 % m.per_part) << m.shift) + (part & ((1 << m.shift) - 1));
    return *tile < ntiles;
}

// the second product of a two-product launch (N < 64 form only; grid.y = 2)
struct GatherSecond {
    const int32_t *sptr;
    const int32_t *out_row;
    const uint32_t *rows;
    const uint32_t *desc;
    const unsigned char *payload;
    const unsigned short *X;
    float *Y;
    int32_t usteps;
};

struct GatherParams {
    const int32_t *sptr;
    const int32_t *out_row;   // original row of stored row t * 16 + m, -1 past the matrix
    const uint32_t *rows;
    const uint32_t *desc;
    const unsigned char *payload;
    const unsigned short *X;
    float *Y;
    int64_t N, ldx, ldy;
    int32_t nbr, ntiles;      // nbr: 16-row runs of the stored row order
    int32_t usteps;           // > 0: steps of every run (sptr is not read)
    int32_t yvec;
    XcdMap map;
    GatherSecond second;
#ifdef GRIM_DBG
    long long *dbg;
#endif
};

#ifdef GRIM_DBG
#define GATHER_STAMP(slot) do { if (p.dbg && (threadIdx.x & 63) == 0 && threadIdx.x < 256) p.dbg[((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * 8 + (slot)] = (long long)__builtin_amdgcn_s_memtime(); } while (0)
#else
#define GATHER_STAMP(slot) do { } while (0)
#endif

// WIDE: rows of X are 16-byte aligned (else 8-byte: two loads per piece); NARROW: N < 64;
// SOLO: strips of a few steps only (a 3 x 3 layer of 64 channels has 5, a dense first layer 1) -- every wave takes a
// (tile, strip) of its own, four consecutive strips per workgroup: no split of K, no partial tiles, no barrier
// EIGHT: eight waves split a strip's steps instead of four (few workgroups, long strips: the 14 x 14 layers)
template <bool BF16, bool WIDE, bool NARROW, bool SOLO, bool EIGHT>
__global__ void __launch_bounds__(EIGHT ? kGatherLongWaves * 64 : 256, EIGHT ? 1024 / (kGatherLongWaves * 64) : 4) bcr_spmm_gather(GatherParams p) {
    constexpr int NWV = EIGHT ? kGatherLongWaves : 4;          // waves of the workgroup
    constexpr int NT = 4, TN = 64, PITCH = 128, CPR = 8;
    constexpr int SB = 4;                        // steps a wave has in flight
    extern __shared__ __attribute__((aligned(16))) char lds[];
    // workgroup -> (tile, stored strip, or four of them for SOLO)
    const int wave0 = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int tile, unit;
    if (!xcd_map_at(p.map, blockIdx.x, p.ntiles, &tile, &unit)) return;
    const int t = SOLO ? unit * 4 + wave0 : unit;
    if (t >= p.nbr) return;                                           // (SOLO has no barrier a wave could be missed at)
    // the matrix and operands of this workgroup: grid.y = 1 selects the second product of a two-product launch
    const int32_t *sptr = p.sptr, *out_row = p.out_row;
    const uint32_t *rows = p.rows, *desc = p.desc;
    const unsigned char *payload = p.payload;
    const unsigned short *X = p.X;
    float *Y = p.Y;
    int usteps = p.usteps;
    if constexpr (NARROW) {
        if (blockIdx.y) {
            sptr = p.second.sptr; out_row = p.second.out_row; rows = p.second.rows; desc = p.second.desc;
            payload = p.second.payload; X = p.second.X; Y = p.second.Y; usteps = p.second.usteps;
        }
    }
    GATHER_STAMP(0);
    int64_t n0 = (int64_t)tile * TN;
    if (n0 + TN > p.N && p.N >= TN) n0 = p.N - TN;   // ragged last tile: overlap the neighbour (N % 4 == 0)
    // N < 64: one tile that starts at column 0; its pieces past N are fetched from column 0 instead (never stored)

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // one dependent memory round trip less at the start when every run has the same number of steps
    const int g0 = usteps ? t * usteps : sptr[t], nst = usteps ? usteps : sptr[t + 1] - g0;
    const int s_beg = SOLO ? g0 : g0 + (int)((int64_t)nst * wave / NWV);
    const int s_end = SOLO ? g0 + nst : g0 + (int)((int64_t)nst * (wave + 1) / NWV);
    char *buf = lds + wave * 8192;               // two step buffers of 32 rows x 128 bytes

    // fetch side: lane = (row slot rs, 16-byte piece c); its i-th load is k slot i * 8 + rs
    const int rs = lane >> 3, c = lane & 7;
    const bool in_a = !NARROW || c * 8 < p.N, in_b = !NARROW || c * 8 + 4 < p.N;
    const unsigned short *xcol = X + n0 + (in_a ? c * 8 : 0);
    const int boff = in_b ? 4 : 0;               // second half of a piece (8-byte aligned rows)
    int wr_off[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int lrow = i * 8 + rs;
        wr_off[i] = lrow * PITCH + ((c ^ swizzle<CPR>(lrow)) << 4);
    }
    // multiply side: lane = (output row m_row, k group); the two transpose reads of a sub-tile
    // name k slots kgroup * 8 + qd and + 4
    const int i16 = lane & 15, kgroup = lane >> 4, qd = i16 >> 2, m_row = i16;
    const unsigned int below = (1u << m_row) - 1u;
    const int ncolb = (4 * (i16 & 3)) * 2, cl = ncolb >> 4, within = ncolb & 15;
    const int r0 = kgroup * 8 + qd, r1 = r0 + 4;
    const int sw0 = swizzle<CPR>(r0), sw1 = swizzle<CPR>(r1);
    const int x0 = r0 * PITCH + within, x1 = r1 * PITCH + within;

    f32x4 acc[NT];
#pragma unroll
    for (int q = 0; q < NT; ++q) acc[q] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int orow = out_row[(int64_t)t * 16 + (lane & 15)];     // asked for now, needed at the very end

    const u32x4 *rows4 = reinterpret_cast<const u32x4 *>(rows);
    const uint2 *desc2 = reinterpret_cast<const uint2 *>(desc);
    const i16x8 *pay = reinterpret_cast<const i16x8 *>(payload);
    // Row numbers and descriptor of the first step of the next batch are asked for together with
    // the current batch's, so that a wave whose steps do not fit one batch (18 steps over 4 waves:
    // 4 + 1) starts the rows of X of the next batch without another dependent round trip.
    u32x4 nhdr = {0u, 0u, 0u, 0u};
    uint2 ndsc = {0u, 0u};
    if (s_beg < s_end) {
        nhdr = rows4[(int64_t)s_beg * 8 + rs];
        ndsc = desc2[(int64_t)s_beg * 4 + kgroup];
    }
    for (int s = s_beg; s < s_end; s += SB) {
        const int nb = s_end - s < SB ? s_end - s : SB;
        u32x4 hdr[SB];
        uint2 dsc[SB];
        hdr[0] = nhdr;
        dsc[0] = ndsc;
#pragma unroll
        for (int u = 1; u < SB; ++u) {
            const int st = s + (u < nb ? u : nb - 1);
            hdr[u] = rows4[(int64_t)st * 8 + rs];
            dsc[u] = desc2[(int64_t)st * 4 + kgroup];
        }
        {
            const int st = s + SB < s_end ? s + SB : s_end - 1;
            nhdr = rows4[(int64_t)st * 8 + rs];
            ndsc = desc2[(int64_t)st * 4 + kgroup];
        }
        u32x4 RX[SB][4];
        i16x8 PW[SB];
#pragma unroll
        for (int u = 0; u < SB; ++u) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const unsigned int row = hdr[u][i] == 0xffffffffu ? 0u : hdr[u][i];
                const unsigned short *src = xcol + (int64_t)row * p.ldx;
                if constexpr (WIDE) {
                    RX[u][i] = *reinterpret_cast<const u32x4 *>(src);
                } else {
                    const uint2 a = *reinterpret_cast<const uint2 *>(src);
                    const uint2 b = *reinterpret_cast<const uint2 *>(NARROW ? src + boff : src + 4);
                    RX[u][i] = u32x4{a.x, a.y, b.x, b.y};
                }
            }
            const bool kept = (dsc[u].x >> m_row) & 1u;
            const unsigned int idx = dsc[u].y + (kept ? __builtin_popcount(dsc[u].x & below) : 0);
            const i16x8 wv = pay[idx];           // a block's first kept row if this lane's is not kept (zeroed below)
            PW[u] = kept ? wv : i16x8{0, 0, 0, 0, 0, 0, 0, 0};
        }
#ifdef GRIM_DBG
        if (s == s_beg) { GATHER_STAMP(1); if (RX[0][0][0] == 0x12345678u && PW[SB - 1][0] == 77) GATHER_STAMP(7); GATHER_STAMP(2); }
#endif
#pragma unroll
        for (int u = 0; u < SB; ++u) {
            if (u < nb) {
                char *b = buf + (u & 1) * 4096;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const u32x4 v = hdr[u][i] == 0xffffffffu ? u32x4{0u, 0u, 0u, 0u} : RX[u][i];
                    *reinterpret_cast<u32x4 *>(b + wr_off[i]) = v;
                }
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int q = 0; q < NT; ++q) {
                    const int cq = q * 2 + cl;
                    const i16x4 lo = lds_tr_read(b + x0 + ((cq ^ sw0) << 4));
                    const i16x4 hi = lds_tr_read(b + x1 + ((cq ^ sw1) << 4));
                    const i16x8 x = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    acc[q] = mfma16<BF16>(x, PW[u], acc[q]);
                }
                __builtin_amdgcn_wave_barrier();
            }
        }
    }

    if constexpr (SOLO) {
        // the wave owns the whole 16 x 64 tile: D[n][m], lane holds m = lane % 16, n = 4 * (lane / 16) + 0..3 of sub-tile q
        const int64_t row = orow;
        if (row >= 0) {
#pragma unroll
            for (int q = 0; q < NT; ++q) {
                const int64_t n = n0 + q * 16 + 4 * (lane >> 4);
                if (n < p.N) {
                    float *dst = Y + row * p.ldy + n;
                    if (p.yvec == 4) {
                        *reinterpret_cast<f32x4 *>(dst) = acc[q];
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) dst[e] = acc[q][e];
                    }
                }
            }
        }
        GATHER_STAMP(6);
        return;
    }
    // add the waves' partial tiles in wave order; wave q finishes sub-tile q.  A wave parks its
    // partial tile in its own (now idle) step buffers.
    GATHER_STAMP(4);
    f32x4 *red = reinterpret_cast<f32x4 *>(lds);
#pragma unroll
    for (int q = 0; q < NT; ++q) red[wave * 512 + q * 64 + lane] = acc[q];
    __syncthreads();
    GATHER_STAMP(5);
    if (EIGHT && wave >= NT) return;             // the first four waves finish the four sub-tiles
    const int q = wave;
    f32x4 sum = red[q * 64 + lane];
#pragma unroll
    for (int w = 1; w < NWV; ++w) {
        const f32x4 v = red[w * 512 + q * 64 + lane];
        sum[0] += v[0]; sum[1] += v[1]; sum[2] += v[2]; sum[3] += v[3];
    }
    // D[n][m]: lane holds m = lane % 16, n = 4 * (lane / 16) + 0..3
    const int64_t row = orow;
    const int64_t n = n0 + q * 16 + 4 * (lane >> 4);
    if (row >= 0 && n < p.N) {                   // n, N multiples of 4: all four columns or none
        float *dst = Y + row * p.ldy + n;
        if (p.yvec == 4) {
            *reinterpret_cast<f32x4 *>(dst) = sum;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) dst[e] = sum[e];
        }
    }
    GATHER_STAMP(6);
}

// Wave per (tile, strip) instead of four waves splitting a strip's steps: strips of at most 8 steps (two batches of a
// wave) with enough pairs to fill the GPU, and longer strips once there are half as many pairs again (measured: 9 steps
// x 1568 pairs 11.3 -> 10.4 us, 18 steps x 12544 pairs 144 -> 129 us; 18 steps x 784 pairs 11.1 -> 12.9 us)
// (the convolution kernel, with more work per step: 9 x 1568 15.4 -> 16.3 us, 18 x 12544 138 -> 113 us; it asks for 4096)
static bool gather_wave_per_strip(const grim_bcr_matrix *A, int64_t pairs, int64_t pairs_for_long_strips = 1536) {
    return (A->gather.max_steps <= 8 && pairs >= 1024) || (A->gather.max_steps <= 40 && pairs >= pairs_for_long_strips);
}

bool gather_applies(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx) {
    return A->gather.present && N >= 4 && N % 4 == 0 && ldx % 4 == 0 && reinterpret_cast<uintptr_t>(X) % 8 == 0;
}

// Bytes through one compute unit, the quantity both matrix-core kernels are bound by at these
// sizes: a workgroup fetches the rows of X its strip keeps (128 bytes each) and the strip's
// records, pays a start-up, and 256 compute units share the workgroups.
double gather_cost(const grim_bcr_matrix *A, int64_t N) {
    const GatherLayout &L = A->gather;
    const double nbr = (double)L.nstrips;
    const double per_wg = (double)L.xrows / nbr * 128.0 + ((double)L.nsteps * 160.0 + (double)L.payload.size()) / nbr;
    const double nwg = (double)((N + 63) / 64) * nbr;
    // the bytes go through the compute units one after the other; the start-up of a workgroup overlaps with the
    // three others a compute unit holds
    return (nwg > 256.0 ? nwg / 256.0 : 1.0) * per_wg + (nwg > 1024.0 ? nwg / 1024.0 : 1.0) * 30e3;
}

// Two products Y = A X and Y2 = A2 X2 of fewer than 64 columns in one launch (the two gate products of a GRU step):
// same element type, number of 16-row runs, N and leading dimensions; K may differ.
bool gather_pair_applies(const grim_bcr_matrix *A, const void *X, const grim_bcr_matrix *A2, const void *X2, int64_t N,
                         int64_t ldx) {
    return N < 64 && gather_applies(A, X, N, ldx) && gather_applies(A2, X2, N, ldx) && A->dtype == A2->dtype &&
           A->gather.nstrips == A2->gather.nstrips;
}

grim_status launch_spmm_gather(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, float *Y, int64_t ldy,
                               hipStream_t stream, const grim_bcr_matrix *A2, const void *X2, float *Y2) {
    if (!gather_applies(A, X, N, ldx)) return GRIM_ERR_UNSUPPORTED;
    if (A2 && !gather_pair_applies(A, X, A2, X2, N, ldx)) return GRIM_ERR_UNSUPPORTED;
    GatherParams p;
    p.sptr = A->gather.d_sptr;
    p.rows = A->gather.d_rows;
    p.desc = A->gather.d_desc;
    p.payload = A->gather.d_payload;
    p.out_row = A->gather.d_out_row;
    p.X = static_cast<const unsigned short *>(X);
    p.Y = Y;
    p.N = N; p.ldx = ldx; p.ldy = ldy;
    p.nbr = (int32_t)A->gather.nstrips;
    p.usteps = A->gather.usteps;
    p.ntiles = (int32_t)((N + 63) / 64);
    p.yvec = (reinterpret_cast<uintptr_t>(Y) % 16 == 0 && ldy % 4 == 0 && N % 4 == 0) ? 4 : 1;
    p.second = GatherSecond{p.sptr, p.out_row, p.rows, p.desc, p.payload, p.X, p.Y, p.usteps};
    if (A2) {
        p.second = GatherSecond{A2->gather.d_sptr, A2->gather.d_out_row, A2->gather.d_rows, A2->gather.d_desc,
                                A2->gather.d_payload, static_cast<const unsigned short *>(X2), Y2, A2->gather.usteps};
        if (reinterpret_cast<uintptr_t>(Y2) % 16 != 0) p.yvec = 1;
    }
    // strips of at most 8 steps (two batches of a wave) with enough (tile, strip) pairs to fill the GPU: wave per pair;
    // long strips and fewer workgroups than compute units: eight waves per strip
    const bool narrow = N < 64;
    const bool solo = !narrow && gather_wave_per_strip(A, (int64_t)p.ntiles * p.nbr);
    const bool eight = !narrow && !solo && A->gather.max_steps >= 16 && (int64_t)p.ntiles * p.nbr <= 256;
    const int64_t per_tile = solo ? (p.nbr + 3) / 4 : p.nbr;
    if (((int64_t)p.ntiles + 7) / 8 * 8 * per_tile > 0x7fffffff) return GRIM_ERR_SHAPE;
    int64_t nwg = 0;
    p.map = xcd_map(p.ntiles, per_tile, &nwg);
    if (nwg > 0x7fffffff) return GRIM_ERR_SHAPE;
#ifdef GRIM_DBG
    p.dbg = reinterpret_cast<long long *>(getenv("GRIM_DBG_PTR") ? strtoull(getenv("GRIM_DBG_PTR"), nullptr, 0) : 0ull);
#endif
    const size_t lds = (eight ? kGatherLongWaves : 4) * 8192;
    const bool wide = N % 8 == 0 && ldx % 8 == 0 && reinterpret_cast<uintptr_t>(X) % 16 == 0 &&
                      (!A2 || reinterpret_cast<uintptr_t>(X2) % 16 == 0);
    const dim3 grid((unsigned)nwg, A2 ? 2u : 1u), block(eight ? kGatherLongWaves * 64 : 256);
#define GRIM_GATHER(BF, WD, NR, SO, EI)                                                                              \
    do {                                                                                                             \
        auto kern = bcr_spmm_gather<BF, WD, NR, SO, EI>;                                                             \
        static std::atomic<bool> attr_done{false};   /* raising a kernel's LDS limit is needed once per process */  \
        if (lds > 64 * 1024 && !attr_done) {                                                                         \
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                    160 * 1024) != hipSuccess) {                                                     \
                (void)hipGetLastError();                                                                             \
                return GRIM_ERR_DEVICE;                                                                              \
            }                                                                                                        \
            attr_done = true;                                                                                        \
        }                                                                                                            \
        hipLaunchKernelGGL(kern, grid, block, lds, stream, p);                                                       \
    } while (0)
#define GRIM_GATHER_DT(BF)                                                                                         \
    if (narrow) { if (wide) GRIM_GATHER(BF, true, true, false, false); else GRIM_GATHER(BF, false, true, false, false); }        \
    else if (solo) { if (wide) GRIM_GATHER(BF, true, false, true, false); else GRIM_GATHER(BF, false, false, true, false); }     \
    else if (eight) { if (wide) GRIM_GATHER(BF, true, false, false, true); else GRIM_GATHER(BF, false, false, false, true); }    \
    else { if (wide) GRIM_GATHER(BF, true, false, false, false); else GRIM_GATHER(BF, false, false, false, false); }
    if (A->dtype == GRIM_BF16) { GRIM_GATHER_DT(true) } else { GRIM_GATHER_DT(false) }
#undef GRIM_GATHER_DT
#undef GRIM_GATHER
    return hipGetLastError() == hipSuccess ? GRIM_OK : GRIM_ERR_DEVICE;
}

// ------------------------------------------------------------------------------------------
// convolution with the im2col matrix never formed (Section 3.1: CONV = filter matrix x im2col
// matrix; Section 4.5: rows of that matrix whose weights are all pruned are skipped)
//
// Same scheme and layout as the row-gathering kernel; only the fetch differs.  Row k of the
// im2col matrix is (input channel cin, kernel row r, kernel column q) with k = cin * kh * kw +
// r * kw + q, and its entry at output position n = h * W + w is F[cin][h + r - kh/2][w + q - kw/2]
// (zero outside the image).  For 8 consecutive positions these are 8 consecutive elements of the
// feature map starting at cin * H * W + n + (r - kh/2) * W + (q - kw/2) -- at any 2-byte alignment
// -- with some of them invalid at the image border.  A lane loads its window with one 16-byte
// load at that address, and when the step is multiplied zeroes the invalid elements with a
// 16-byte mask that depends on (kernel tap, piece of the tile) only and is read from a table the
// workgroup builds in LDS when it starts.  A window that would reach outside the feature map
// (the first and last few positions of the first and last channel) is put together from single
// guarded element loads instead.  Only rows kept by the strip are ever touched, and the feature
// map is read instead of a matrix kh * kw times its size.
// ------------------------------------------------------------------------------------------
struct ConvParams {
    const int32_t *sptr;
    const int32_t *out_row;
    const uint32_t *rows;
    const uint32_t *desc;
    const unsigned char *payload;
    const unsigned short *F;     // [Cin][H][W]
    void *Y;                     // [M][ldy] of fp32, fp16 or bf16 (odt), position n = h * W + w
    const float *bias;           // [M] added to every position of a row, or null
    int64_t ldy;
    int32_t odt, relu;           // element type of Y; max(., 0) after the bias
    int32_t N, H, W, kh, kw;     // N = H * W
    int32_t KK, kk_magic;        // kh * kw and ceil(2^31 / KK): k / KK = umulhi(2 k, magic) while k * KK < 2^31 (checked at launch)
    int32_t kw_magic;            // ceil(256 / kw): tap / kw = tap * magic >> 8 (checked for every tap at launch)
    int32_t total;               // elements of the feature map
    int32_t nbr, ntiles;
    int32_t usteps;              // > 0: steps of every run (sptr is not read)
    int32_t yvec;
    XcdMap map;
};

// fp32 -> bf16, round to nearest even; NaN stays NaN
__device__ __forceinline__ unsigned short conv_f32_to_bf16(float f) {
    unsigned int u = __builtin_bit_cast(unsigned int, f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

struct __attribute__((packed, aligned(4))) ConvWindow {
    unsigned int d[4];
};

constexpr int kConvMaxTaps = 31;   // 5 bits of the packed (tap, window start) word, one value left for padding slots
constexpr int kConvTableBytes = (kConvMaxTaps + 1) * 8 * 16;   // validity masks, behind the waves' step buffers

// SOLO, EIGHT: as in the row-gathering kernel -- a (tile, strip) pair per wave for strips of a few steps, eight
// waves per strip for long strips with few workgroups
template <bool BF16, bool SOLO, int LONGW>   // LONGW: 0, or the waves that split a long strip's steps (8 or 12)
__global__ void __launch_bounds__(LONGW ? LONGW * 64 : 256, LONGW ? 1024 / (LONGW * 64) : 4) bcr_conv_gather(ConvParams p) {
    constexpr bool EIGHT = LONGW > 0;
    constexpr int NT = 4, TN = 64, PITCH = 128, CPR = 8;
    constexpr int SB = 3;                        // steps a wave has in flight
    constexpr int NWV = EIGHT ? LONGW : 4;       // waves of the workgroup
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int tile, unit;
    if (!xcd_map_at(p.map, blockIdx.x, p.ntiles, &tile, &unit)) return;
    const int t_raw = SOLO ? unit * 4 + wave : unit;
    const bool active = t_raw < p.nbr;           // SOLO: the last workgroup of a tile may have idle waves
    const int t = active ? t_raw : p.nbr - 1;
    int n0 = tile * TN;
    if (n0 + TN > p.N) n0 = p.N - TN;            // ragged last tile: overlap the neighbour
    n0 = n0 < 0 ? 0 : n0;                        // a map of fewer than 64 positions: one tile, its columns past N never stored

    // one dependent memory round trip less at the start when every run has the same number of steps
    const int g0 = p.usteps ? t * p.usteps : p.sptr[t], nst = p.usteps ? p.usteps : p.sptr[t + 1] - g0;
    const int s_beg = SOLO ? g0 : g0 + (int)((int64_t)nst * wave / NWV);
    const int s_end = SOLO ? g0 + nst : g0 + (int)((int64_t)nst * (wave + 1) / NWV);
    char *buf = lds + wave * 8192;
    // The first batch's row numbers and block descriptors are asked for before the validity table is built,
    // so that their latency runs under it.
    const int kgroup0 = lane >> 4;
    const uint2 *desc2 = reinterpret_cast<const uint2 *>(p.desc);
    unsigned int npk[SB];
    uint2 ndsc[SB];
#pragma unroll
    for (int u = 0; u < SB; ++u) {
        int st = s_beg + u;
        st = st < s_end ? st : s_end - 1;
        st = st < 0 ? 0 : st;                    // (a wave without steps: any valid step, never used)
        npk[u] = p.rows[(int64_t)st * 32 + (lane & 7) * 4 + ((lane >> 3) & 3)];
        ndsc[u] = desc2[(int64_t)st * 4 + kgroup0];
    }
    // per (tap, piece of the tile) the 16-byte validity mask of the piece's 8 positions; entry KK
    // is all zero (padding slots).
    u32x4 *vtab = reinterpret_cast<u32x4 *>(lds + NWV * 8192);
    const int ph = p.kh >> 1, pw = p.kw >> 1;
    if (tid < (p.KK + 1) * 8) {
        const int tap = tid >> 3, cc = tid & 7;
        const int r = tap / p.kw, q = tap - r * p.kw;
        const int dr = r - ph, dq = q - pw;
        const int nb = n0 + cc * 8;
        const int h0 = nb / p.W, w0 = nb - h0 * p.W;
        unsigned int m[4] = {0u, 0u, 0u, 0u};
        if (tap < p.KK) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                int h = h0, w = w0 + j;
                while (w >= p.W) { w -= p.W; ++h; }  // once at most for W >= 8 (positions past N, of a small map: h >= H, never stored)
                const bool ok = h + dr >= 0 && h + dr < p.H && w + dq >= 0 && w + dq < p.W;
                m[j >> 1] |= ok ? (j & 1 ? 0xffff0000u : 0x0000ffffu) : 0u;
            }
        }
        vtab[tid] = u32x4{m[0], m[1], m[2], m[3]};
    }
    __syncthreads();
    if (SOLO && !active) return;                 // (no barrier follows in that form)

    // fetch side: lane = (row slot rs, piece c): positions n0 + 8 c .. n0 + 8 c + 7 of the tile
    const int rs = lane >> 3, c = lane & 7;
    const int wr_off0 = rs * PITCH + ((c ^ swizzle<CPR>(rs)) << 4);     // the swizzle does not depend on i (row i * 8 + rs)
    // multiply side (as in the row-gathering kernel)
    const int i16 = lane & 15, kgroup = lane >> 4, qd = i16 >> 2, m_row = i16;
    const unsigned int below = (1u << m_row) - 1u;
    const int ncolb = (4 * (i16 & 3)) * 2, cl = ncolb >> 4, within = ncolb & 15;
    const int r0 = kgroup * 8 + qd, r1 = r0 + 4;
    const int sw0 = swizzle<CPR>(r0), sw1 = swizzle<CPR>(r1);
    const int x0 = r0 * PITCH + within, x1 = r1 * PITCH + within;
    // the lane's two transpose reads of sub-tile 0
    const unsigned int buf_lds = (unsigned int)(uintptr_t)(__attribute__((address_space(3))) char *)buf;
    const unsigned int tr0 = x0 + ((cl ^ sw0) << 4), tr1 = x1 + ((cl ^ sw1) << 4);           // offsets in a step buffer

    f32x4 acc[NT];
#pragma unroll
    for (int q = 0; q < NT; ++q) acc[q] = f32x4{0.f, 0.f, 0.f, 0.f};

    const i16x8 *pay = reinterpret_cast<const i16x8 *>(p.payload);
    const char *Fb = reinterpret_cast<const char *>(p.F);
    const int HW = p.N, wstep = p.W - p.kw, emax = p.total - 8;
    const int nshift0 = n0 - (ph * p.W + pw);    // window start relative to a channel, tile's first column, centre tap removed
    const int cofs = c * 8 - (1 << 25);          // this lane's piece, and the bias of the packed form
    // can a window of this tile start before the feature map or end behind it?  (only in the first / last channel)
    const bool tile_edge = n0 < ph * p.W + pw || n0 + TN + ph * p.W + pw > HW;
    for (int s = s_beg; s < s_end; s += SB) {
        const int nb = s_end - s < SB ? s_end - s : SB;
        // Lane j takes k slot j % 32 of every step of the batch: it splits the slot's row number once into
        // (window start for the tile's first column, tap) and the lanes that fetch the slot's eight row
        // pieces pick that pair up with a lane permute -- one integer division per lane and step instead of
        // four.  Packed as tap (or KK for padding) << 27 | window start + 2^25.
        unsigned int pk[SB];
        uint2 dsc[SB];
#pragma unroll
        for (int u = 0; u < SB; ++u) {
            if (s == s_beg) {
                pk[u] = npk[u];
                dsc[u] = ndsc[u];
            } else {
                const int st = s + (u < nb ? u : nb - 1);
                pk[u] = p.rows[(int64_t)st * 32 + (lane & 7) * 4 + ((lane >> 3) & 3)];
                dsc[u] = desc2[(int64_t)st * 4 + kgroup];
            }
        }
        u32x4 RX[SB][4];
        unsigned int vsel[SB];                   // per step, 8 bits per window: validity mask (the tap; KK: padding) | odd start << 7
        i16x8 PW[SB];
        unsigned int ext[SB];
        // window start of piece (u, i) for this lane, and the selector of its validity mask
        auto piece = [&](int u, int i, unsigned int &sel) {
            const unsigned int v = (unsigned int)__shfl((int)pk[u], i * 8 + rs);
            sel = v >> 27;
            return (int)(v & 0x7ffffffu) + cofs;
        };
        // SAFE: the tile touches the first or last positions of the feature map, where a window can reach
        // outside it (first / last channel only); every other tile skips those checks altogether.
        auto fetch = [&](auto safe_tag) {
            constexpr bool SAFE = decltype(safe_tag)::value;
#pragma unroll
            for (int u = 0; u < SB; ++u) {
                const bool is_pad = pk[u] == 0xffffffffu;
                const unsigned int kk = is_pad ? 0u : pk[u];
                // (24-bit multiplies: Cin, H * W, W and the tap numbers are all below 2^24)
                const unsigned int cin = __umulhi(kk << 1, (unsigned int)p.kk_magic);
                const int tap = (int)(kk - __umul24(cin, (unsigned int)p.KK));
                const unsigned int r = __umul24((unsigned int)tap, (unsigned int)p.kw_magic) >> 8;   // tap / kw
                // r * W + (tap - r * kw), less the centre tap's offset, for the tile's first column
                const int eb = (int)__umul24(cin, (unsigned int)HW) + __mul24((int)r, wstep) + tap + nshift0;   // (W < kw: wstep < 0)
                pk[u] = (unsigned int)(is_pad ? p.KK : tap) << 27 | (unsigned int)(eb + (1 << 25));
                // A 16-byte load at an odd element (2 bytes off a dword) costs about three aligned ones in the
                // vector L1, a load that is only dword-aligned next to nothing.  A window that starts at an odd
                // element is therefore fetched one element early; when the step is written the lane shifts it
                // by 16 bits and takes its last element from the next lane's first dword.  The last lane of a
                // row piece has no such neighbour: lanes 0..31 fetch the boundary element of their k slot with
                // one extra 2-byte load per step, handed over by a lane permute.
                const int e7 = eb + 56;
                bool need = lane < 32 && !is_pad && (e7 & 1);
                if constexpr (SAFE) need = need && e7 + 7 >= 0 && e7 + 7 < p.total;
                ext[u] = need ? (unsigned int)p.F[e7 + 7] : 0u;
            }
            bool edge_any = false;
#pragma unroll
            for (int u = 0; u < SB; ++u) {
                vsel[u] = 0u;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    unsigned int sel;
                    const int e0 = piece(u, i, sel);
                    const int odd = e0 & 1;
                    vsel[u] |= (sel | (unsigned int)odd << 7) << (8 * i);
                    int ea = e0 - odd;
                    if constexpr (SAFE) {
                        const bool edge = e0 < 0 || e0 > emax;
                        edge_any |= edge;
                        ea = edge ? 0 : ea;
                    }
                    ConvWindow wv;
                    __builtin_memcpy(&wv, Fb + (unsigned int)(ea * 2), 16);      // byte offset below 2^31
                    RX[u][i] = u32x4{wv.d[0], wv.d[1], wv.d[2], wv.d[3]};
                }
            }
            if constexpr (SAFE) {
                if (__builtin_amdgcn_ballot_w64(edge_any)) {
#pragma unroll
                    for (int u = 0; u < SB; ++u) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            unsigned int sel;
                            const int e0 = piece(u, i, sel);
                            if (e0 < 0 || e0 > emax) {
                                // the same eight elements the common path fetches (one early for an odd start), so
                                // that the lane's neighbours find what they expect in its first dword
                                unsigned int d[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                                for (int j = 0; j < 8; ++j) {
                                    const int e = e0 - (e0 & 1) + j;
                                    const unsigned int v = e >= 0 && e < p.total ? p.F[e] : 0u;
                                    d[j >> 1] |= v << ((j & 1) * 16);
                                }
                                RX[u][i] = u32x4{d[0], d[1], d[2], d[3]};
                            }
                        }
                    }
                }
            }
        };
        if (tile_edge) fetch(std::true_type{}); else fetch(std::false_type{});
#pragma unroll
        for (int u = 0; u < SB; ++u) {
            const bool kept = (dsc[u].x >> m_row) & 1u;
            const unsigned int idx = dsc[u].y + (kept ? __builtin_popcount(dsc[u].x & below) : 0);
            const i16x8 wv = pay[idx];
            PW[u] = kept ? wv : i16x8{0, 0, 0, 0, 0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < SB; ++u) {
            if (u < nb) {
                char *b = buf + (u & 1) * 4096;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const unsigned int sel = (vsel[u] >> (8 * i)) & 0xffu;
                    const u32x4 vm = vtab[(sel & 0x7fu) * 8 + c];
                    const unsigned int sh = (sel >> 7) * 16u;             // 16: the window starts one element into the fetch
                    // the dword after the lane's four: the next lane's first one, or the boundary element
                    const unsigned int w0 = RX[u][i][0];
                    const unsigned int nxt = (unsigned int)__builtin_amdgcn_update_dpp(0, (int)w0, 0x101 /* row_shl:1 */, 0xf, 0xf, true);
                    const unsigned int bnd = (unsigned int)__shfl((int)ext[u], i * 8 + rs);
                    const unsigned int w4 = c == 7 ? bnd : nxt;
                    const u32x4 v = {__builtin_amdgcn_alignbit(RX[u][i][1], w0, sh) & vm[0],
                                     __builtin_amdgcn_alignbit(RX[u][i][2], RX[u][i][1], sh) & vm[1],
                                     __builtin_amdgcn_alignbit(RX[u][i][3], RX[u][i][2], sh) & vm[2],
                                     __builtin_amdgcn_alignbit(w4, RX[u][i][3], sh) & vm[3]};
                    *reinterpret_cast<u32x4 *>(b + wr_off0 + i * 8 * PITCH) = v;
                }
                __builtin_amdgcn_wave_barrier();
                // The 16-byte chunk of sub-tile q is (2 q + cl) ^ swizzle = (cl ^ swizzle) ^ 2 q: the eight
                // read addresses are two bases with q << 5 XOR-ed in.  The empty asm keeps the compiler from
                // holding all eight in registers across the loop (they would not fit and spill).
                unsigned int a0 = tr0, a1 = tr1;
                asm volatile("" : "+v"(a0), "+v"(a1));
                const unsigned int sb = buf_lds + (u & 1) * 4096;
#pragma unroll
                for (int q = 0; q < NT; ++q) {
                    const i16x4 lo = lds_tr_read_at(sb + (a0 ^ (unsigned int)(q << 5)));
                    const i16x4 hi = lds_tr_read_at(sb + (a1 ^ (unsigned int)(q << 5)));
                    const i16x8 x = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    acc[q] = mfma16<BF16>(x, PW[u], acc[q]);
                }
                __builtin_amdgcn_wave_barrier();
            }
        }
    }

    // epilogue of a layer for four consecutive positions n .. n + 3 of output channel `row`: bias, rectifier,
    // rounding to the next layer's element type
    auto finish = [&](int64_t row, int64_t n, f32x4 sum) {
        const float b = p.bias ? p.bias[row] : 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            sum[e] += b;
            if (p.relu) sum[e] = sum[e] > 0.f ? sum[e] : 0.f;     // NaN stays NaN
        }
        const bool vec = p.yvec == 4 && (n & 3) == 0;
        const int left = (int)(p.N - n);             // below 4 only in the one tile of a map of fewer than 64 positions
        if (p.odt == GRIM_F32) {
            float *dst = static_cast<float *>(p.Y) + row * p.ldy + n;
            if (vec && left >= 4) {
                *reinterpret_cast<f32x4 *>(dst) = sum;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (e < left) dst[e] = sum[e];
            }
        } else {
            unsigned short h[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (p.odt == GRIM_F16) {
                    const _Float16 v = (_Float16)sum[e];
                    __builtin_memcpy(&h[e], &v, 2);
                } else {
                    h[e] = conv_f32_to_bf16(sum[e]);
                }
            }
            unsigned short *dst = static_cast<unsigned short *>(p.Y) + row * p.ldy + n;
            if (vec && left >= 4) {
                *reinterpret_cast<uint2 *>(dst) = uint2{(unsigned int)h[0] | ((unsigned int)h[1] << 16), (unsigned int)h[2] | ((unsigned int)h[3] << 16)};
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (e < left) dst[e] = h[e];
            }
        }
    };
    const int64_t row = p.out_row[(int64_t)t * 16 + (lane & 15)];
    if constexpr (SOLO) {
        if (row >= 0) {
#pragma unroll
            for (int q = 0; q < NT; ++q) finish(row, n0 + q * 16 + 4 * (lane >> 4), acc[q]);
        }
        return;
    }
    // the waves' partial tiles go through their step buffers; the tables behind them stay intact
    f32x4 *red = reinterpret_cast<f32x4 *>(lds);
#pragma unroll
    for (int q = 0; q < NT; ++q) red[wave * 512 + q * 64 + lane] = acc[q];
    __syncthreads();
    if (EIGHT && wave >= NT) return;             // the first four waves finish the four sub-tiles
    const int q = wave;
    f32x4 sum = red[q * 64 + lane];
#pragma unroll
    for (int w = 1; w < NWV; ++w) {
        const f32x4 v = red[w * 512 + q * 64 + lane];
        sum[0] += v[0]; sum[1] += v[1]; sum[2] += v[2]; sum[3] += v[3];
    }
    if (row >= 0) finish(row, n0 + q * 16 + 4 * (lane >> 4), sum);
}

grim_status launch_conv_gather(const grim_bcr_matrix *A, const void *F, int32_t Cin, int32_t H, int32_t W, int32_t kh,
                               int32_t kw, const float *bias, int32_t relu, void *Y, int32_t odt, int64_t ldy,
                               hipStream_t stream) {
    const int64_t N = (int64_t)H * W, total = (int64_t)Cin * N;
    if (!A->gather.present || total < 8 || kh * kw > kConvMaxTaps || total > (int64_t(1) << 26) || (int64_t)(kh / 2) * W + kw / 2 >= (1 << 24) ||
        A->K > (int64_t(1) << 27) || A->K * (int64_t)(kh * kw) > (int64_t(1) << 31) || Cin >= (1 << 24) || N >= (1 << 24) || reinterpret_cast<uintptr_t>(F) % 2 != 0)
        return GRIM_ERR_UNSUPPORTED;
    ConvParams p;
    p.sptr = A->gather.d_sptr;
    p.out_row = A->gather.d_out_row;
    p.rows = A->gather.d_rows;
    p.desc = A->gather.d_desc;
    p.payload = A->gather.d_payload;
    p.F = static_cast<const unsigned short *>(F);
    p.Y = Y;
    p.bias = bias;
    p.odt = odt;
    p.relu = relu;
    p.ldy = ldy;
    p.N = (int32_t)N; p.H = H; p.W = W; p.kh = kh; p.kw = kw;
    p.KK = kh * kw;
    p.kk_magic = (int32_t)(uint32_t)(((uint64_t(1) << 31) + p.KK - 1) / p.KK);
    p.kw_magic = (256 + kw - 1) / kw;
    for (int tap = 0; tap < p.KK; ++tap)
        if (((tap * p.kw_magic) >> 8) != tap / kw) return GRIM_ERR_UNSUPPORTED;   // (1 x 25 and the like)
    p.total = (int32_t)total;
    p.nbr = (int32_t)A->gather.nstrips;
    p.usteps = A->gather.usteps;
    p.ntiles = (int32_t)((N + 63) / 64);
    // four consecutive outputs of a row in one store: 16 bytes of fp32, 8 bytes of fp16 / bf16
    p.yvec = (reinterpret_cast<uintptr_t>(Y) % (odt == GRIM_F32 ? 16 : 8) == 0 && ldy % 4 == 0 && N % 4 == 0) ? 4 : 1;
    // the same launch forms as the row-gathering kernel
    const bool solo = gather_wave_per_strip(A, (int64_t)p.ntiles * p.nbr, 4096);
    const int64_t pairs = (int64_t)p.ntiles * p.nbr;
    // long strips and few pairs: twelve waves per strip up to 256 pairs (one workgroup per compute unit), eight up to 512
    // (two per compute unit; 28 x 28 layers: 11.0 -> 9.4 us with 18 steps, 14.1 -> 13.3 us with 36)
    const int longw = !solo && A->gather.max_steps >= 16 ? (pairs <= 256 ? kConvLongWaves : pairs <= 512 ? 8 : 0) : 0;
    const int64_t per_tile = solo ? (p.nbr + 3) / 4 : p.nbr;
    if (((int64_t)p.ntiles + 7) / 8 * 8 * per_tile > 0x7fffffff) return GRIM_ERR_SHAPE;
    int64_t nwg = 0;
    p.map = xcd_map(p.ntiles, per_tile, &nwg);
    if (nwg > 0x7fffffff) return GRIM_ERR_SHAPE;
    const size_t lds = (size_t)(longw ? longw : 4) * 8192 + kConvTableBytes;
    const dim3 grid((unsigned)nwg), block(longw ? longw * 64 : 256);
#define GRIM_CONV(BF, SO, EI)                                                                                        \
    do {                                                                                                             \
        auto kern = bcr_conv_gather<BF, SO, EI>;                                                                     \
        static std::atomic<bool> attr_done{false};                                                                   \
        if (lds > 64 * 1024 && !attr_done) {                                                                         \
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                    160 * 1024) != hipSuccess) {                                                     \
                (void)hipGetLastError();                                                                             \
                return GRIM_ERR_DEVICE;                                                                              \
            }                                                                                                        \
            attr_done = true;                                                                                        \
        }                                                                                                            \
        hipLaunchKernelGGL(kern, grid, block, lds, stream, p);                                                       \
    } while (0)
    if (A->dtype == GRIM_BF16) { if (solo) GRIM_CONV(true, true, 0); else if (longw == 12) GRIM_CONV(true, false, 12); else if (longw == 8) GRIM_CONV(true, false, 8); else GRIM_CONV(true, false, 0); }
    else { if (solo) GRIM_CONV(false, true, 0); else if (longw == 12) GRIM_CONV(false, false, 12); else if (longw == 8) GRIM_CONV(false, false, 8); else GRIM_CONV(false, false, 0); }
#undef GRIM_CONV
    return hipGetLastError() == hipSuccess ? GRIM_OK : GRIM_ERR_DEVICE;
}

bool mma_supported(const grim_bcr_matrix *A) { return A->mma.present; }

static int amax_of(const grim_bcr_matrix *A, int g) { return A->mma.amax[g <= 4 ? 0 : g <= 8 ? 1 : g <= 16 ? 2 : 3]; }

// Compiled launch shapes.  Groups of 4 strips use 4 consumer waves, larger groups 8 (LDS reads
// per MFMA are high, so a second consumer wave per SIMD hides their latency); always 8
// producer waves (two teams of 4), each holding SX slots of X and SR slots of records.
struct MmaShape { int tn, strips, nw, sx, sr; };
static bool mma_shape(int BR, int tn, int strips, MmaShape *out) {
    const int sx = tn == 32 ? 4 : tn == 64 ? 8 : tn == 128 ? 16 : 0;      // 256 staged rows
    const int sr = strips == 4 ? 4 : strips == 8 ? 8 : strips == 16 ? 12 : 0;
    if (!sx || !sr) return false;
    if (tn == 128 && strips != 4) return false;
    const int nw = strips == 4 ? 4 : 8;
    if (BR == 32 && (strips / nw) * (tn / 32) > 4) return false;           // accumulator registers
    *out = MmaShape{tn, strips, nw, sx, sr};
    return true;
}
static bool mma_shape_fits(const grim_bcr_matrix *A, int tn, int strips) {
    MmaShape sh;
    if (!mma_shape(A->BR, tn, strips, &sh)) return false;
    const int rps = 1024 / (tn * 2), amax = amax_of(A, strips);
    if ((A->mma.chunk_rows + rps - 1) / rps > 4 * sh.sx) return false;
    if ((amax * 16 + 1023) / 1024 > 4 * sh.sr) return false;
    return 2 * (int64_t)mma_stage_bytes(A->mma.chunk_rows, tn * 2, amax) + (int64_t)A->mma.nchunks * (strips + 1) * 8 <= 160 * 1024;
}

template <bool BF16, int BR, int NT, int SPW, int NW, int SX, int SR>
static grim_status launch_mma_inst(const MmaParams &p, hipStream_t stream) {
    constexpr int TN = NT * (BR == 16 ? 16 : 32);
    const size_t lds = 2 * (size_t)mma_stage_bytes(p.chunk_rows, TN * 2, p.amax) + (size_t)p.nchunks * (NW * SPW + 1) * 8;
    const int64_t tiles8 = ((int64_t)p.ntiles + 7) / 8 * 8;
    const int64_t nwg = tiles8 * p.ngroups;
    if (nwg > 0x7fffffff) return GRIM_ERR_SHAPE;
    auto kern = bcr_spmm_mma<BF16, BR, NT, SPW, NW, 8, SX, SR>;
    static std::atomic<bool> attr_done{false};    // raising a kernel's LDS limit is needed once per process
    if (lds > 64 * 1024 && !attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) {
            (void)hipGetLastError();
            return GRIM_ERR_DEVICE;
        }
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3((NW + 8) * 64), lds, stream, p);
    return hipGetLastError() == hipSuccess ? GRIM_OK : GRIM_ERR_DEVICE;
}

template <bool BF16, int BR>
static grim_status launch_mma_br(MmaParams &p, const grim_bcr_matrix *A, int tile_n, int strips, hipStream_t stream) {
    constexpr int NSUB = BR == 16 ? 16 : 32;
    p.ntiles = (int32_t)((p.N + tile_n - 1) / tile_n);
    p.ngroups = (p.nbr + strips - 1) / strips;
    p.amax = amax_of(A, strips);
#define GRIM_CASE(TN_, G_, NW_, SX_, SR_) \
    if (tile_n == TN_ && strips == G_) return launch_mma_inst<BF16, BR, TN_ / NSUB, G_ / NW_, NW_, SX_, SR_>(p, stream);
#ifdef GRIM_FEW_SHAPES   /* development builds: two shapes */
    GRIM_CASE(64, 4, 4, 8, 4) GRIM_CASE(64, 16, 8, 8, 12)
#else
    GRIM_CASE(32, 4, 4, 4, 4) GRIM_CASE(32, 8, 8, 4, 8) GRIM_CASE(32, 16, 8, 4, 12)
    GRIM_CASE(64, 4, 4, 8, 4) GRIM_CASE(64, 8, 8, 8, 8) GRIM_CASE(64, 16, 8, 8, 12)
    GRIM_CASE(128, 4, 4, 16, 4)
#endif
#undef GRIM_CASE
    return GRIM_ERR_UNSUPPORTED;
}

// Pick the launch shape by bytes through one compute unit: a workgroup streams its tile's rows of
// X (64-byte row pieces of a 32-column tile cost about 1.8x per byte), the records of its strips,
// and pays a fixed start-up (130 KB worth: two barriers' worth of pipeline fill); workgroups beyond 256 run in rounds.  Returns the cost (< 0: no
// compiled shape fits); tile_n / strips_per_wg != 0 pin that knob.
double mma_best_shape(const grim_bcr_matrix *A, int64_t N, int32_t tile_n, int32_t strips_per_wg, int *tn_out, int *g_out) {
    if (!A->mma.present) return -1.0;
    const double rec_total = (double)A->mma.recs.size();
    double best = -1.0;
    for (int t : {64, 32}) {
        if (tile_n && t != tile_n) continue;
        for (int g : {16, 8, 4}) {
            if (strips_per_wg && g != strips_per_wg) continue;
            if (g > 4 && A->nbr <= g / 2) continue;
            if (!mma_shape_fits(A, t, g)) continue;
            const int64_t nwg = ((N + t - 1) / t) * ((A->nbr + g - 1) / g);
            const double rounds = (double)((nwg + 255) / 256);
            const double bytes = (double)A->K * t * 2 * (t == 32 ? 1.8 : 1.0) +
                                 rec_total * (double)(g < A->nbr ? g : A->nbr) / (double)A->nbr + 130e3;
            const double cost = rounds * bytes;
            if (best < 0 || cost < best) { best = cost; *tn_out = t; *g_out = g; }
        }
    }
    return best;
}

// The staged kernel's workgroups are large (one or two fit a compute unit), so a launch runs in rounds of that many
// workgroups and a few left over cost a whole round: 784 tiles on 256 compute units take 4 rounds for 3.06 rounds of
// work.  Returns the number of leading columns that fill whole rounds (a multiple of the tile width) and the launch
// shape for them when, by the cost model that also picks the kernel, these plus the remaining columns as a product of
// their own (on the row-gathering kernel if `rest_may_gather`, else staged again) come cheaper than one launch; the
// caller sends the remaining columns through the kernel choice.  Returns N when there is nothing to gain.
int64_t mma_whole_rounds(const grim_bcr_matrix *A, int64_t N, bool rest_may_gather, int *tn_out, int *g_out) {
    int tn = 0, g = 0;
    const double cost_all = mma_best_shape(A, N, 0, 0, &tn, &g);
    if (cost_all < 0) return N;
    *tn_out = tn; *g_out = g;
    const int64_t ntiles = (N + tn - 1) / tn, ngroups = (A->nbr + g - 1) / g;
    const int64_t lds = 2 * (int64_t)mma_stage_bytes(A->mma.chunk_rows, tn * 2, amax_of(A, g)) + (int64_t)A->mma.nchunks * (g + 1) * 8;
    const int threads = ((g == 4 ? 4 : 8) + 8) * 64;
    int64_t per_cu = 160 * 1024 / lds;
    if (per_cu > 2048 / threads) per_cu = 2048 / threads;
    if (per_cu < 1) per_cu = 1;
    const int64_t slots = 256 * per_cu, nwg = ntiles * ngroups;
    const int64_t full = nwg / slots * slots, rest = nwg - full;
    if (full == 0 || rest == 0 || full % ngroups != 0) return N;
    const int64_t n_main = full / ngroups * tn, n_rest = N - n_main;
    int t2 = 0, g2 = 0;
    const double cost_main = mma_best_shape(A, n_main, tn, g, &t2, &g2);
    double cost_rest = mma_best_shape(A, n_rest, 0, 0, &t2, &g2);
    if (rest_may_gather && A->gather.present) {
        const double c = gather_cost(A, n_rest);
        if (cost_rest < 0 || c < cost_rest) cost_rest = c;
    }
    if (cost_main < 0 || cost_rest < 0 || cost_main + cost_rest > 0.97 * cost_all) return N;
    return n_main;
}

grim_status launch_spmm_mma(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, float *Y, int64_t ldy,
                            int32_t tile_n, int32_t strips_per_wg, hipStream_t stream) {
    if (!A->mma.present) return GRIM_ERR_UNSUPPORTED;
    if (tile_n != 0 && tile_n != 32 && tile_n != 64 && tile_n != 128) return GRIM_ERR_UNSUPPORTED;
    if (strips_per_wg != 0 && strips_per_wg != 4 && strips_per_wg != 8 && strips_per_wg != 16) return GRIM_ERR_UNSUPPORTED;
    int tn = tile_n, strips = strips_per_wg;
    if (!tn || !strips) {
        if (mma_best_shape(A, N, tile_n, strips_per_wg, &tn, &strips) < 0) return GRIM_ERR_UNSUPPORTED;
    }
    if (!mma_shape_fits(A, tn, strips)) return GRIM_ERR_UNSUPPORTED;
    MmaParams p;
    p.recs = A->mma.d_recs;
    p.cptr = A->mma.d_cptr;
    p.bptr = A->mma.d_bptr;
    p.strip_order = A->dev.strip_order;
    p.X = static_cast<const unsigned short *>(X);
    p.Y = Y;
    p.N = N; p.ldx = ldx; p.ldy = ldy;
    p.K = (int32_t)A->K; p.nbr = (int32_t)A->nbr; p.nchunks = A->mma.nchunks; p.chunk_rows = A->mma.chunk_rows;
    const uintptr_t xa = reinterpret_cast<uintptr_t>(X), ya = reinterpret_cast<uintptr_t>(Y);
    p.xvec = (xa % 16 == 0 && ldx % 8 == 0) ? 8 : (xa % 8 == 0 && ldx % 4 == 0) ? 4 : 1;
    p.yvec = (ya % 16 == 0 && ldy % 4 == 0) ? 4 : 1;
#ifdef GRIM_DBG
    p.dbg = reinterpret_cast<long long *>(getenv("GRIM_DBG_PTR") ? strtoull(getenv("GRIM_DBG_PTR"), nullptr, 0) : 0ull);
#endif
    const bool bf = A->dtype == GRIM_BF16;
    if (A->BR == 16) return bf ? launch_mma_br<true, 16>(p, A, tn, strips, stream) : launch_mma_br<false, 16>(p, A, tn, strips, stream);
    return bf ? launch_mma_br<true, 32>(p, A, tn, strips, stream) : launch_mma_br<false, 32>(p, A, tn, strips, stream);
}

}  // namespace grim

#include "spmm_common.hpp"

namespace grim {

// Row-gathering matrix-core SpMM kernel for Y = W_bcr * X (Section 3.1; Section 4.4: the rows of X a block
// keeps are loaded once and reused by all of its kept rows).
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
    int32_t K;                // rows of X
    int32_t touch;            // start the tile's rows of X on their way from HBM when the workgroup starts
    XcdMap map;
    GatherSecond second;
};


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
    int64_t n0 = (int64_t)tile * TN;
    if (n0 + TN > p.N && p.N >= TN) n0 = p.N - TN;   // ragged last tile: overlap the neighbour (N % 4 == 0)
    // N < 64: one tile that starts at column 0; its pieces past N are fetched from column 0 instead (never stored)

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // A wave learns which rows of X it needs only after a first round trip (row numbers), and fetches them in one or
    // two batches: with X in HBM that is up to three dependent trips to memory.  The strips of a tile run at the same
    // time on one XCD and together keep nearly every row of the tile (16 strips keeping a quarter each leave 1 % out),
    // so each workgroup starts its share of ALL the tile's rows on their way into that XCD's L2 right now -- one byte
    // from the first and the last 128-byte line of every row piece, values never used -- and the fetches proper find
    // them there or on their way.
    if constexpr (!NARROW) {
        if (p.touch) {
            const int units = p.map.per_tile;                          // workgroups of this tile
            const int per = (p.K + units - 1) / units;
            const int r_end = (unit + 1) * per < p.K ? (unit + 1) * per : p.K;
            const char *base = reinterpret_cast<const char *>(X + n0) + (tid & 1) * 127;
            for (int r = unit * per + (tid >> 1); r < r_end; r += NWV * 32)
                (void)*reinterpret_cast<const volatile unsigned char *>(base + (int64_t)r * p.ldx * 2);
        }
    }
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
        return;
    }
    // add the waves' partial tiles in wave order; wave q finishes sub-tile q.  A wave parks its
    // partial tile in its own (now idle) step buffers.
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
}

// Wave per (tile, strip) instead of four waves splitting a strip's steps: strips of at most 8 steps (two batches of a
// wave) with enough pairs to fill the GPU, and longer strips once there are half as many pairs again (measured: 9 steps
// x 1568 pairs 11.3 -> 10.4 us, 18 steps x 12544 pairs 144 -> 129 us; 18 steps x 784 pairs 11.1 -> 12.9 us)
// (the convolution kernel, with more work per step: 9 x 1568 15.4 -> 16.3 us, 18 x 12544 138 -> 113 us; it asks for 4096)
bool gather_wave_per_strip(const grim_bcr_matrix *A, int64_t pairs, int64_t pairs_for_long_strips) {
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
    p.K = (int32_t)A->K;
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
    // Long strips only: a wave then runs ten and more dependent batches, and having the rows in L2 shortens each (the
    // last 512 columns of a 4608-row product: 10 -> 7.7 us); with 18-step strips the extra requests cost more than they
    // save (12.0 -> 12.4 us on a 2304-row product, five-step strips 15.5 -> 24 us).
    p.touch = !narrow && A->gather.max_steps >= 40 ? 1 : 0;
    const bool solo = !narrow && gather_wave_per_strip(A, (int64_t)p.ntiles * p.nbr, 1536);
    const bool eight = !narrow && !solo && A->gather.max_steps >= 16 && (int64_t)p.ntiles * p.nbr <= 256;
    const int64_t per_tile = solo ? (p.nbr + 3) / 4 : p.nbr;
    if (((int64_t)p.ntiles + 7) / 8 * 8 * per_tile > 0x7fffffff) return GRIM_ERR_SHAPE;
    int64_t nwg = 0;
    p.map = xcd_map(p.ntiles, per_tile, &nwg);
    if (nwg > 0x7fffffff) return GRIM_ERR_SHAPE;
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


}  // namespace grim

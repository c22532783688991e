// Kernel of bcr_spmm_gather.hip as a header: the wide-tile kernel's launcher builds a kernel that runs both.
#pragma once
#include <type_traits>

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


// which form of the kernel a launch takes, and its workgroups
struct GatherForm {
    bool wide, narrow, solo, eight;
    int64_t nwg;
};
grim_status gather_setup(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, float *Y, int64_t ldy,
                         const grim_bcr_matrix *A2, const void *X2, float *Y2, GatherParams *out, GatherForm *form);

// WIDE: rows of X are 16-byte aligned (else 8-byte: two loads per piece); NARROW: N < 64;
// SOLO: strips of a few steps only (a 3 x 3 layer of 64 channels has 5, a dense first layer 1) -- every wave takes a
// (tile, strip) of its own, four consecutive strips per workgroup: no split of K, no partial tiles, no barrier
// EIGHT: eight waves split a strip's steps instead of four (few workgroups, long strips: the 14 x 14 layers)
// The body of the kernel as a function of the workgroup's number (block_x; block_y: second product of a pair), so that
// another kernel can run such workgroups next to its own (the wide-tile kernel does, for the columns it leaves over).
// Its first NWV waves must call it together; `lds` = NWV * 8 KB of workgroup memory.
// LONGW: the waves that split a strip in the EIGHT form (eight in the kernel of its own; a caller with more waves to
// spare may pass more: fewer steps per wave, fewer dependent batches).
template <bool BF16, bool WIDE, bool NARROW, bool SOLO, bool EIGHT, int LONGW = kGatherLongWaves>
__device__ __forceinline__ void gather_body(const GatherParams &p, char *lds, int block_x, int block_y) {
    constexpr int NWV = EIGHT ? LONGW : 4;                     // waves of the workgroup
    constexpr int NT = 4, TN = 64, PITCH = 128, CPR = 8;
    constexpr int SB = 4;                        // steps a wave has in flight
    // workgroup -> (tile, stored strip, or four of them for SOLO)
    const int wave0 = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int tile, unit;
    if (!xcd_map_at(p.map, block_x, p.ntiles, &tile, &unit)) return;
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
        if (block_y) {
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
    // The rows of X of a step (pad: bit i set = the lane's i-th k slot is padding and multiplies zeros; kept instead of
    // the row numbers) and its weights, asked for into a register set
    struct StepRows { u32x4 rx[4]; unsigned int pad; };
    auto ask_rows = [&](StepRows &r, const u32x4 &h) {
        r.pad = 0u;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            r.pad |= h[i] == 0xffffffffu ? 1u << i : 0u;
            const unsigned int row = h[i] == 0xffffffffu ? 0u : h[i];
            const unsigned short *src = xcol + (int64_t)row * p.ldx;
            if constexpr (WIDE) {
                r.rx[i] = *reinterpret_cast<const u32x4 *>(src);
            } else {
                const uint2 a = *reinterpret_cast<const uint2 *>(src);
                const uint2 b = *reinterpret_cast<const uint2 *>(NARROW ? src + boff : src + 4);
                r.rx[i] = u32x4{a.x, a.y, b.x, b.y};
            }
        }
    };
    auto ask_weights = [&](const uint2 &d) {
        const bool kept = (d.x >> m_row) & 1u;
        const unsigned int idx = d.y + (kept ? __builtin_popcount(d.x & below) : 0);
        const i16x8 wv = pay[idx];               // a block's first kept row if this lane's is not kept (zeroed below)
        return kept ? wv : i16x8{0, 0, 0, 0, 0, 0, 0, 0};
    };
    // A batch: SB steps in flight.  The rows of the first step of the NEXT batch are asked for as soon as this batch's
    // first step has left its registers -- its row numbers came with this batch's -- so that a wave with one step more
    // than a batch holds (18 steps over 4 waves: 4 + 1) does not pay a whole further round trip for it: the request
    // travels while the rest of this batch arrives (FIRST: the batch that finds nothing asked for yet).  (With the
    // request made unconditional in a copy of the batch for "another batch follows", so that every wait counts exactly
    // the younger loads, the compiler needs 158 registers for what takes 128 here: not done.)
    StepRows early;
    auto batch = [&](int s, auto first_tag) {
        constexpr bool FIRST = decltype(first_tag)::value;
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
        StepRows R[SB];
        i16x8 PW[SB];
        if constexpr (!FIRST) R[0] = early;      // asked for during the batch before
#pragma unroll
        for (int u = 0; u < SB; ++u) {
            if (FIRST || u > 0) ask_rows(R[u], hdr[u]);
            PW[u] = ask_weights(dsc[u]);
        }
#pragma unroll
        for (int u = 0; u < SB; ++u) {
            if (u < nb) {
                char *b = buf + (u & 1) * 4096;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const u32x4 v = (R[u].pad >> i) & 1u ? u32x4{0u, 0u, 0u, 0u} : R[u].rx[i];
                    *reinterpret_cast<u32x4 *>(b + wr_off[i]) = v;
                }
                __builtin_amdgcn_wave_barrier();
                if (u == 0 && s + SB < s_end) ask_rows(early, nhdr);   // set 0's rows are out of their registers
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
    };
    if (s_beg < s_end) batch(s_beg, std::true_type{});
    for (int s = s_beg + SB; s < s_end; s += SB) batch(s, std::false_type{});

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

template <bool BF16, bool WIDE, bool NARROW, bool SOLO, bool EIGHT>
__global__ void __launch_bounds__(EIGHT ? kGatherLongWaves * 64 : 256, EIGHT ? 1024 / (kGatherLongWaves * 64) : 4) bcr_spmm_gather(GatherParams p) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    gather_body<BF16, WIDE, NARROW, SOLO, EIGHT>(p, lds, blockIdx.x, blockIdx.y);
}

}  // namespace grim

// Staged matrix-core SpMM kernel (fp16 / bf16, BR = 16 or 32) for Y = W_bcr * X (Section 3.1).
// A workgroup owns a tile of TN columns of X and a group of row strips.  Chunks of consecutive X rows are
// staged in LDS once per workgroup (tiling, Section 4.4) by dedicated producer waves (global -> registers ->
// LDS), two chunks ahead of the consumer waves.  Each consumer wave gathers the rows its strips keep with LDS
// transpose reads straight into MFMA operand layout and multiplies them with the kept rows of the blocks'
// weights (lanes of rows a block does not keep multiply zeros).  Strips are dealt to waves in stored
// (work-sorted, Section 4.2) order so the waves of a workgroup carry near-equal work.  Accumulation is fp32,
// order fixed, no atomics.
#include "spmm_common.hpp"

namespace grim {

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
};


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
        if (team < p.nchunks) load_chunk(team, false);        // team 0: chunk 0, team 1: chunk 1
        if (team == 0) store_chunk(0, false);
        __syncthreads();
        for (int j = 0; j < p.nchunks; ++j) {
            if ((j & 1) == team) {
                if (j + 2 < p.nchunks) load_chunk(j + 2, true);   // registers were emptied one chunk ago
            } else {
                if (j + 1 < p.nchunks) store_chunk(j + 1, true);  // stage (j + 1) % 2 was read last in chunk j - 1
            }
            __syncthreads();
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
#pragma unroll
        for (int s = 0; s < SPW; ++s) en[s] = en_next[s];
        __syncthreads();
    }

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
    GRIM_CASE(32, 4, 4, 4, 4) GRIM_CASE(32, 8, 8, 4, 8) GRIM_CASE(32, 16, 8, 4, 12)
    GRIM_CASE(64, 4, 4, 8, 4) GRIM_CASE(64, 8, 8, 8, 8) GRIM_CASE(64, 16, 8, 8, 12)
    GRIM_CASE(128, 4, 4, 16, 4)
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
    const bool bf = A->dtype == GRIM_BF16;
    if (A->BR == 16) return bf ? launch_mma_br<true, 16>(p, A, tn, strips, stream) : launch_mma_br<false, 16>(p, A, tn, strips, stream);
    return bf ? launch_mma_br<true, 32>(p, A, tn, strips, stream) : launch_mma_br<false, 32>(p, A, tn, strips, stream);
}


}  // namespace grim

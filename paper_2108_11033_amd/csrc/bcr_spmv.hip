// SpMV / skinny SpMM kernel: y = W_bcr * x for 1..8 right-hand sides (Section 3.1: FC and
// RNN gate layers are matrix-vector products).
//
// The compact weights ARE the memory traffic here, so they are read exactly once, in their
// compact kept-rows x kept-columns form (Section 4.3), with 8 bytes of row / column bit masks
// per block as the only index data.  Matrices whose blocks all keep the same counts go to the
// wave-per-strip kernels further down (bcr_spmv_wave_exact for one right-hand side,
// bcr_spmv_wave_exact_b for several in a large launch); everything else to bcr_spmv, where one
// workgroup owns one row strip:
//   1. the strip's weights -- one contiguous byte range -- its block masks and x are fetched with
//      coalesced 16-byte loads, all issued before any is used, and parked in LDS;
//   2. a group of LPB lanes takes a block, lane i its compact row i: a dot product over the
//      block's kept columns with x gathered from LDS (every gathered x value is shared by all kept
//      rows of the block -- the load-redundancy elimination of Section 4.4); partial sums go to
//      private LDS slots;
//   3. one thread per (strip row, right-hand side, block range) adds the partials of the blocks
//      that keep its row in ascending block order, then the block ranges are added in ascending
//      order: a fixed summation tree, no atomics, bit-reproducible.
// Strips too large for LDS are processed in segments of column blocks.
#include <hip/hip_runtime.h>

#include <atomic>

#include <cstdlib>

#include "bcr_matrix.hpp"
#include "spmv_common.hpp"

namespace grim {

// threads of a workgroup of bcr_spmv: from 2 right-hand sides on, twice as many lanes share the strip's blocks and
// outputs (the phases are chains of dependent LDS round trips, so more waves per strip shorten them)
__host__ __device__ constexpr int gemv_threads(int B) { return B >= 2 ? 512 : 256; }

template <int DT, int B, int VEC>
__global__ void __launch_bounds__(gemv_threads(B), (B == 1 ? 6 : 1)) bcr_spmv(GemvParams p) {
    constexpr int NTH = gemv_threads(B);
    using T = typename GElem<DT>::type;
    struct __attribute__((aligned(sizeof(T) * VEC))) WVec { T v[VEC]; };
    struct __attribute__((aligned(sizeof(T) * VEC))) XVec { T v[VEC * B]; };
    extern __shared__ __attribute__((aligned(16))) char smem[];
    // LDS: [weights segment + 16][row masks][column masks][block offsets][gathered x per block]
    //      [partials + one zero slot][block-range sums][x]
    char *wl = smem;
    unsigned int *rmask = reinterpret_cast<unsigned int *>(smem + p.wbytes + 16);
    unsigned int *cmask = rmask + kSegMax;
    unsigned int *wof = cmask + kSegMax;
    const int xgs = gemv_xg_stride(p.kcmax, B);
    T *xg = reinterpret_cast<T *>(wof + kSegMax + 4);                      // [seg_blocks][xgs]
    float *part = reinterpret_cast<float *>(reinterpret_cast<char *>(xg) + ((p.seg_blocks * xgs * (int)sizeof(T) + 15) & ~15));
    const int zero_slot = p.seg_blocks * p.krmax * B;                      // part[zero_slot] == 0
    float *red = part + ((zero_slot + 4) & ~3);                            // [nseg][BR * B]
    const int rb = p.BR * B;                                               // outputs of the strip
    const int nseg = NTH / rb;                                             // BR <= 32 and B <= 8: rb <= 256
    T *xs = reinterpret_cast<T *>(red + ((nseg * rb + 3) & ~3));

    const int tid = threadIdx.x;
    const int64_t t = blockIdx.x;            // stored strip
    const int64_t mi = blockIdx.y;           // matrix of the group
    const GemvGlobal d = to_global(p.table ? p.table[mi] : mi ? p.second : p.single);
    const GRIM_GLOBAL char *W = d.weights;
    const GRIM_GLOBAL T *x = (const GRIM_GLOBAL T *)p.x + mi * p.x_stride;
    GRIM_GLOBAL float *y = (GRIM_GLOBAL float *)p.y + mi * p.y_stride;
    const int lpb = 1 << p.lpb_shift;

    // reducer role: thread -> (block range sg, output o = r * B + b)
    const int sg = tid / rb, o = tid % rb;
    const int r_out = o / B, b_out = o % B;
    const bool reducer = sg < nseg;
    float yacc = 0.f;
    if (tid == 0) part[zero_slot] = 0.f;

    for (int c0 = 0; c0 < p.nbc; c0 += p.seg_blocks) {
        const int nb = p.nbc - c0 < p.seg_blocks ? p.nbc - c0 : p.seg_blocks;
        const int64_t blk0 = t * p.nbc + c0;
        // ---- 1. fetch: block masks / offsets, the segment's weights, and (first segment) x;
        //         every load is issued before any is used ----
        unsigned int m0 = 0, m1 = 0, wo = 0;
        if (tid < nb) {
            const gu32x2 mm = *reinterpret_cast<const GRIM_GLOBAL gu32x2 *>(d.masks + 2 * (blk0 + tid));
            m0 = mm.x;
            m1 = mm.y;
        }
        unsigned int wstart, wend;           // element range of the segment's weights
        if (p.ukr >= 0) {
            wstart = (unsigned int)blk0 * (unsigned int)(p.ukr * p.ukc);
            wend = wstart + (unsigned int)nb * (unsigned int)(p.ukr * p.ukc);
            if (tid <= nb) wo = wstart + (unsigned int)tid * (unsigned int)(p.ukr * p.ukc);
        } else {
            wstart = d.woff[blk0];
            wend = d.woff[blk0 + nb];
            if (tid <= nb) wo = d.woff[blk0 + tid];
        }
        const unsigned int bstart = wstart * (unsigned int)sizeof(T), bend = wend * (unsigned int)sizeof(T);
        const unsigned int a0 = bstart & ~15u;               // 16-byte aligned fetch window
        const int nvec = (int)((bend - a0 + 15u) >> 4);      // <= kWLoads * 256 by construction
        // round 0 of the weights and of x share one latency; later rounds (large segments, wide x)
        // are rare and run one after the other
        const bool xfast = c0 == 0 && p.xvec16;
        const int nxv = xfast ? p.K * B / (16 / (int)sizeof(T)) : 0;
        const GRIM_GLOBAL gu32x4 *xsrc = reinterpret_cast<const GRIM_GLOBAL gu32x4 *>(x);
        gu32x4 wreg[4], xreg[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (i * NTH < nvec) {                            // same for the whole workgroup
                int v = tid + i * NTH;
                v = v < nvec ? v : nvec - 1;                 // clamp: the duplicates are never stored
                wreg[i] = *reinterpret_cast<const GRIM_GLOBAL gu32x4 *>(W + a0 + (size_t)v * 16);
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (i * NTH < nxv) {
                int v = tid + i * NTH;
                v = v < nxv ? v : nxv - 1;
                xreg[i] = xsrc[v];
            }
        }
        if (c0 > 0) __syncthreads();                          // previous segment fully consumed
        if (tid < nb) { rmask[tid] = m0; cmask[tid] = m1; }
        if (tid <= nb) wof[tid] = wo - wstart;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int v = tid + i * NTH;
            if (v < nvec) *reinterpret_cast<gu32x4 *>(wl + (size_t)v * 16) = wreg[i];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int v = tid + i * NTH;
            if (v < nxv) reinterpret_cast<gu32x4 *>(xs)[v] = xreg[i];
        }
        for (int v = tid + 4 * NTH; v < nvec; v += NTH)
            *reinterpret_cast<gu32x4 *>(wl + (size_t)v * 16) = *reinterpret_cast<const GRIM_GLOBAL gu32x4 *>(W + a0 + (size_t)v * 16);
        for (int v = tid + 4 * NTH; v < nxv; v += NTH) reinterpret_cast<gu32x4 *>(xs)[v] = xsrc[v];
        if (c0 == 0 && !p.xvec16) {
            // x with a leading dimension or unaligned: element by element, layout [k][b]
            for (int e = tid; e < p.K * B; e += NTH) xs[e] = x[(int64_t)(e / B) * p.ldx + (e % B)];
        }
        __syncthreads();
        // ---- 2. lane group -> block.  The group first gathers the block's kept columns of x
        //         (lane li takes kept columns li, li + lpb, ...); group and block live in one
        //         wave, whose LDS operations complete in order, so no workgroup barrier is needed
        //         before the rows read the gathered values.  Then lane -> compact row: dot product.
        const T *wbase = reinterpret_cast<const T *>(wl + (bstart - a0));
        const int slots = NTH >> p.lpb_shift;
        const int li = tid & (lpb - 1);
        for (int s = tid >> p.lpb_shift; s < nb; s += slots) {
            const unsigned int cm = cmask[s];
            const int kr = __builtin_popcount(rmask[s]), kc = __builtin_popcount(cm);
            T *xgb = xg + s * xgs;
            {
                // kept column j of the block = position of the j-th set bit of its column mask
                const T *xb = xs + (c0 + s) * p.BC * B;
                for (int j = li; j < kc; j += lpb) {
                    const int col = nth_set_bit(cm, j);
#pragma unroll
                    for (int b = 0; b < B; ++b) xgb[j * B + b] = xb[col * B + b];
                }
            }
            __builtin_amdgcn_wave_barrier();
            for (int i = li; i < kr; i += lpb) {
                const T *wr = wbase + wof[s] + i * kc;
                float acc[B];
#pragma unroll
                for (int b = 0; b < B; ++b) acc[b] = 0.f;
#pragma unroll 4
                for (int j = 0; j < kc; j += VEC) {
                    const WVec wv = *reinterpret_cast<const WVec *>(wr + j);
                    const XVec xv = *reinterpret_cast<const XVec *>(xgb + j * B);
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        const float w = g2f<DT>(wv.v[v]);
#pragma unroll
                        for (int b = 0; b < B; ++b) acc[b] = __builtin_fmaf(w, g2f<DT>(xv.v[v * B + b]), acc[b]);
                    }
                }
#pragma unroll
                for (int b = 0; b < B; ++b) part[(s * p.krmax + i) * B + b] = acc[b];
            }
        }
        __syncthreads();
        // ---- 3. per output: add the partials of the blocks that keep its row, ascending ----
        if (reducer) {
            const int per = (nb + nseg - 1) / nseg;
            const int s0 = sg * per, s1 = s0 + per < nb ? s0 + per : nb;
            const unsigned int below = (1u << r_out) - 1u;
            for (int sb = s0; sb < s1; sb += 8) {
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {                 // eight independent LDS reads in flight
                    const int s = sb + u < s1 ? sb + u : s1 - 1;
                    const unsigned int m = rmask[s];
                    const int i = __builtin_popcount(m & below);
                    const bool hit = sb + u < s1 && ((m >> r_out) & 1u);
                    v[u] = part[hit ? (s * p.krmax + i) * B + b_out : zero_slot];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) yacc += v[u];     // adding 0 for a miss changes nothing
            }
        }
    }
    // block ranges are combined in ascending order by the first range's threads
    if (nseg > 1) {
        if (reducer) red[sg * rb + o] = yacc;
        __syncthreads();
        if (tid < rb) {
            float sum = red[o];
            for (int g = 1; g < nseg; ++g) sum += red[g * rb + o];
            yacc = sum;
        }
    }
    if (tid < rb) {
        const int64_t row = (int64_t)d.strip_order[t] * p.BR + r_out;
        y[row * p.ldy + b_out] = yacc;
    }
}

// ------------------------------------------------------------------------------------------
// One right-hand side, every block keeping exactly KR rows and KC columns (a layer pruned at one
// rate): the wave-per-strip scheme with every size known at compile time.
//   - a block is NV 16-byte vectors; the strip's vectors are parked in LDS with a little
//     padding so that 16-byte reads at a fixed offset from the lanes' block bases hit all
//     banks evenly;
//   - a lane reads its whole block and its KC activations into registers; two-byte types
//     multiply pairs with the packed dot-product instruction (fp32 sum, subnormals kept);
//   - each lane scatters its rows' sums to a [strip row][block] table in LDS (zero where a block
//     does not keep the row); lanes (strip row, group) then add each row's 64 entries in a fixed order.
// ------------------------------------------------------------------------------------------
// KEEP: finished strips a lane group holds back before it stores them (see below)
template <int DT, int KR, int KC, int CELL = 0, int KEEP = 4>
__global__ void __launch_bounds__(exact_waves(CELL) * 64) bcr_spmv_wave_exact(GemvParams p) {
    using T = typename GElem<DT>::type;
    constexpr int ESZ = (int)sizeof(T);
    constexpr int NWV = exact_waves(CELL), NTHR = NWV * 64;
    constexpr int NV = KR * KC * ESZ / 16;       // 16-byte vectors per block
    constexpr int PB = exact_pad_period(NV);     // one vector of padding after every PB blocks (0: none)
    static_assert(KR * KC * ESZ % 16 == 0 && (ESZ == 4 || KC % 2 == 0) && KC <= 32 && KR <= 32, "block shape");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // GRU: both input vectors sit in LDS, the hidden-side one behind the input-side one
    const int xsk = exact_x_skew(p.BC, ESZ);     // elements of padding behind every block's part of x (0 or 4 bytes)
    const int xbytes1 = ((p.K + p.nbc * xsk) * ESZ + 15) & ~15, xbytes = CELL == 2 ? 2 * xbytes1 : xbytes1;
    // Several right-hand sides: a set of workgroups per column of x (grid.z; with a cell grid.y), each column on its
    // own compute units -- a matrix of 128 strips is 32 workgroups
    const int bq = CELL != 0 ? blockIdx.y : blockIdx.z;
    const int64_t mi = CELL == 2 ? wave / 3 : CELL == 1 ? 0 : blockIdx.y;   // GRU: waves 0-2 take W_i, waves 3-5 W_h
    T *xs = reinterpret_cast<T *>(smem + (CELL == 2 ? (int)mi * xbytes1 : 0));
    char *wl = smem + xbytes + wave * p.wbytes;
    float *part = reinterpret_cast<float *>(wl);                  // reuses the weights' space

    const GemvGlobal d = to_global(p.table ? p.table[mi] : mi ? p.second : p.single);
    const GRIM_GLOBAL char *W = d.weights;
    const GRIM_GLOBAL T *x = (const GRIM_GLOBAL T *)p.x + (CELL == 2 ? 0 : mi * p.x_stride) + bq;
    GRIM_GLOBAL float *y = (GRIM_GLOBAL float *)p.y + mi * p.y_stride + bq;

    const int nsegs = (p.nbc + p.seg_blocks - 1) / p.seg_blocks;
    // the product alone: a wave walks sps consecutive stored strips; with a cell: the strip of gate `gate` that holds
    // hidden units blockIdx.x * BR .., wherever the reorder has stored it
    const int gate = CELL == 2 ? wave % 3 : wave;
    // (a small launch leaves strips to one or two waves of a workgroup and takes more workgroups: a wave's 12 KB of
    // weights then arrive through a compute unit of their own; the other waves only help to copy x)
    const int wpg = CELL != 0 ? NWV : p.wpg;
    int64_t t0 = ((int64_t)blockIdx.x * wpg + wave) * p.sps;
    if constexpr (CELL != 0) {
        const int32_t *pos = (CELL == 2 && mi) ? p.cell.strip_pos2 : p.cell.strip_pos;
        const int s = gate * (p.cell.H / p.BR) + (int)blockIdx.x;
        t0 = pos ? pos[s] : s;                                    // (no table: stored in the original order)
    }
    const int nstrips = CELL != 0 ? 1 : wave >= wpg ? 0 : p.nbr_total - t0 < p.sps ? (int)(p.nbr_total - t0) : p.sps;   // <= 0: nothing to do
    const int nitems = nstrips > 0 ? nstrips * nsegs : 0;

    struct Item {
        unsigned int rm, cm;
        int nvec, c0, srow;
    };
    gu32x4 wreg[NV];
    auto fetch = [&](int it, Item &I) {
        const int sn = it / nsegs;
        const int sg = it - sn * nsegs;
        const int64_t t = t0 + sn;
        I.c0 = sg * p.seg_blocks;
        const int nb = p.nbc - I.c0 < p.seg_blocks ? p.nbc - I.c0 : p.seg_blocks;
        const int64_t blk0 = t * p.nbc + I.c0;
        I.nvec = nb * NV;
        // the masks first and without a branch: loads return in order, and x can be gathered as soon as the column
        // mask is here, while the weights are still on their way
        const gu32x2 mm = *reinterpret_cast<const GRIM_GLOBAL gu32x2 *>(d.masks + 2 * (blk0 + (lane < nb ? lane : nb - 1)));
        const GRIM_GLOBAL char *src = W + (size_t)blk0 * (NV * 16);
        if (nb == 64) {
#pragma unroll
            for (int i = 0; i < NV; ++i)
                wreg[i] = *reinterpret_cast<const GRIM_GLOBAL gu32x4 *>(src + (unsigned int)(lane * 16 + i * 1024));
        } else {
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                int v = lane + i * 64;
                v = v < I.nvec ? v : I.nvec - 1;
                wreg[i] = *reinterpret_cast<const GRIM_GLOBAL gu32x4 *>(src + (unsigned int)(v * 16));
            }
        }
        I.rm = lane < nb ? mm.x : 0u;
        I.cm = lane < nb ? mm.y : KC == 32 ? 0xffffffffu : (1u << (KC & 31)) - 1u;   // idle lanes: any KC columns, no rows
        I.srow = sg == nsegs - 1 ? d.strip_order[t] : 0;
    };

    // output lanes: (strip row, lane group); 4 groups of 16 lanes up to 16 strip rows, else 2 of 32
    const int ngrp = p.BR <= 16 ? 4 : 2;
    const int r_out = p.BR <= 16 ? lane & 15 : lane & 31;
    const int grp = p.BR <= 16 ? lane >> 4 : lane >> 5;
    // Finished strips wait in registers -- lane group g keeps the strips numbered g, g + ngrp, ...
    // since the last store -- and go out kKeep * ngrp strips at a time, or when the wave is done:
    // few, large stores, whole cache lines when the strips are neighbours in the original order
    // as well (as equal-work strips are), and for launches of one round of workgroups all at the
    // end, where they no longer cut into the stream of weight reads: 16 KB of y scattered into 1.7 MB
    // of reads per product cost 5 % of the time (the same stores into one cache-resident 16 KB cost
    // nothing: it is the DRAM turning round for them).  A large batched launch therefore runs as ONE round of
    // workgroups whose waves walk 16 strips and hold all of them back (KEEP = 8): 0.70 -> 0.745 of
    // HBM peak on 256 products of 4096 x 2048.  Small launches keep 4: the longer run of predicated stores costs a
    // lone product 0.2 us.
    constexpr int kKeep = KEEP;
    float yacc = 0.f, ysum = 0.f, ykeep[kKeep];
    int rowkeep[kKeep], npend = 0;                                // npend: strips kept, not yet stored
    auto store_kept = [&]() {
#pragma unroll
        for (int k = 0; k < kKeep; ++k) {
            if (grp + k * ngrp < npend && r_out < p.BR) y[((int64_t)rowkeep[k] * p.BR + r_out) * p.ldy] = ykeep[k];
        }
        npend = 0;
    };
    // the cell's operands (previous state, biases) are asked for first: their latency runs under the whole product
    float cell_st = 0.f, cell_b[6] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if constexpr (CELL != 0) {
        if (tid < p.BR) {
            const RnnCell &cl = p.cell;
            const int64_t H = cl.H, j = (int64_t)blockIdx.x * p.BR + tid;
            cell_st = cl.c[j * cl.ldc + bq];
#pragma unroll
            for (int k = 0; k < (CELL == 1 ? 4 : 3); ++k) {
                if (cl.bias) cell_b[k] = cl.bias[k * H + j];
                if (CELL == 2 && cl.bias2) cell_b[3 + k] = cl.bias2[k * H + j];
            }
        }
    }
    // x -> LDS, once per workgroup.  Its loads go out first and the first item's right behind
    // them, so that the weights are already on their way while x is parked.
    Item cur, nxt;
    T *xs0 = reinterpret_cast<T *>(smem);                          // (the whole x area: one vector, or two for the GRU)
    const int nvecs = CELL == 2 ? 2 : 1;
    if (p.xvec16) {
        const int nxv1 = p.K * ESZ / 16, nxv = nxv1 * nvecs;
        const GRIM_GLOBAL gu32x4 *xsrc = reinterpret_cast<const GRIM_GLOBAL gu32x4 *>(x);
        const GRIM_GLOBAL gu32x4 *xsrc2 = reinterpret_cast<const GRIM_GLOBAL gu32x4 *>(x + p.x_stride);
        auto src_of = [&](int v) { return v < nxv1 ? xsrc + v : xsrc2 + (v - nxv1); };
        // unit u of a vector goes 4 bytes further for every block before its own: four 4-byte stores
        const int upb = p.BC * ESZ / 16;                           // 16-byte units per block (padded layout only)
        auto put = [&](int v, const gu32x4 &val) {
            const int u = v < nxv1 ? v : v - nxv1;
            unsigned int *dst = reinterpret_cast<unsigned int *>(reinterpret_cast<char *>(xs0) + (v < nxv1 ? 0 : xbytes1)) +
                                u * 4 + (xsk ? u / upb : 0);
            dst[0] = val[0];
            dst[1] = val[1];
            dst[2] = val[2];
            dst[3] = val[3];
        };
        gu32x4 xreg[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (i * NTHR < nxv) {
                int v = tid + i * NTHR;
                v = v < nxv ? v : nxv - 1;
                xreg[i] = *src_of(v);
            }
        if (nitems) fetch(0, cur);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int v = tid + i * NTHR;
            if (v < nxv) put(v, xreg[i]);
        }
        for (int v = tid + 4 * NTHR; v < nxv; v += NTHR) {
            const gu32x4 val = *src_of(v);
            put(v, val);
        }
    } else {
        if (nitems) fetch(0, cur);
        // strided vector(s), element by element: eight loads per thread in flight, then their stores
        const int nel = p.K * nvecs;
        T *xs1 = reinterpret_cast<T *>(reinterpret_cast<char *>(xs0) + xbytes1);
        const int bc_shift = (p.BC & (p.BC - 1)) == 0 ? __builtin_ctz(p.BC) : -1;   // (a power of two: no division per element)
        for (int e0 = tid; e0 < nel; e0 += 8 * NTHR) {
            T v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                int e = e0 + i * NTHR;
                e = e < nel ? e : nel - 1;
                v[i] = e < p.K ? x[(int64_t)e * p.ldx] : x[p.x_stride + (int64_t)(e - p.K) * p.ldx];
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int e = e0 + i * NTHR;
                if (e < nel) {
                    const int k = e < p.K ? e : e - p.K;
                    (e < p.K ? xs0 : xs1)[k + (xsk ? (bc_shift >= 0 ? k >> bc_shift : k / p.BC) * xsk : 0)] = v[i];
                }
            }
        }
    }
    __syncthreads();
    if (!nitems) return;
    for (int it = 0; it < nitems; ++it) {
        const unsigned int rm = cur.rm, cm = cur.cm;
        // this block's KC activations: they need the column mask only, which arrives ahead of the weights
        T xe[KC];
        {
            int xblk = cur.c0 + lane;
            xblk = xblk < p.nbc ? xblk : p.nbc - 1;
            const T *xb = xs + xblk * (p.BC + xsk);
            unsigned int m = cm;
#pragma unroll
            for (int j = 0; j < KC; ++j) {
                const int col = __builtin_ctz(m);                 // KC bits are set
                m &= m - 1;
                xe[j] = xb[col];
            }
        }
        if (cur.nvec == 64 * NV) {
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const int v = lane + i * 64;
                const int slot = PB ? v + v / (NV * PB) : v;
                *reinterpret_cast<gu32x4 *>(wl + slot * 16) = wreg[i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const int v = lane + i * 64;
                const int slot = PB ? v + v / (NV * PB) : v;
                if (v < cur.nvec) *reinterpret_cast<gu32x4 *>(wl + slot * 16) = wreg[i];
            }
        }
        __builtin_amdgcn_wave_barrier();
        // Stores and loads complete in no fixed order relative to each other, so waiting for a
        // load means waiting for every store issued before that wait as well.  The kept sums are
        // therefore stored here, right after the wait for this item's weights and a whole item
        // ahead of the next such wait.
        if (npend == kKeep * ngrp) store_kept();
        nxt = cur;
        if (it + 1 < nitems) fetch(it + 1, nxt);

        gu32x4 w[NV];
        {
            const gu32x4 *wb = reinterpret_cast<const gu32x4 *>(wl) + lane * NV + (PB ? lane / PB : 0);
#pragma unroll
            for (int j = 0; j < NV; ++j) w[j] = wb[j];
        }
        float acc[KR];
        if constexpr (DT == GRIM_F32) {
#pragma unroll
            for (int i = 0; i < KR; ++i) {
                float a = 0.f;
#pragma unroll
                for (int j = 0; j < KC; ++j) {
                    const int q = i * KC + j;
                    const unsigned int wd = w[q >> 2][q & 3];       // a copy: bit_cast of the element itself reads element 0
                    a = __builtin_fmaf(__builtin_bit_cast(float, wd), xe[j], a);
                }
                acc[i] = a;
            }
        } else {
            unsigned int xp[KC / 2];
#pragma unroll
            for (int h = 0; h < KC / 2; ++h) {
                unsigned short lo, hi;
                __builtin_memcpy(&lo, &xe[2 * h], 2);
                __builtin_memcpy(&hi, &xe[2 * h + 1], 2);
                xp[h] = (unsigned int)lo | ((unsigned int)hi << 16);
            }
#pragma unroll
            for (int i = 0; i < KR; ++i) {
                float a = 0.f;
#pragma unroll
                for (int h = 0; h < KC / 2; ++h) {
                    const int q = i * (KC / 2) + h;
                    const unsigned int wd = w[q >> 2][q & 3];
                    if constexpr (DT == GRIM_F16)
                        a = __builtin_amdgcn_fdot2(__builtin_bit_cast(gh2, wd), __builtin_bit_cast(gh2, xp[h]), a, false);
                    else
                        a = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(gb2, wd), __builtin_bit_cast(gb2, xp[h]), a, false);
                }
                acc[i] = a;
            }
        }
        __builtin_amdgcn_wave_barrier();                          // every lane holds its block in registers
        for (int z = lane; z < (p.BR * kPartStride + 3) / 4; z += 64)
            reinterpret_cast<gu32x4 *>(part)[z] = gu32x4{0u, 0u, 0u, 0u};
        __builtin_amdgcn_wave_barrier();
        if (rm) {
            unsigned int m = rm;
#pragma unroll
            for (int i = 0; i < KR; ++i) {
                const int r = __builtin_ctz(m);                   // KR bits are set
                m &= m - 1;
                part[r * kPartStride + lane] = acc[i];
            }
        }
        __builtin_amdgcn_wave_barrier();
        // Row sums in a fixed order.  Up to 16 strip rows: lanes (row, quarter) add 16 blocks
        // each, then quarters pair up; more rows: lanes (row, half) add 32 blocks each.  Every
        // lane group ends up with the full sum.
        float rs;
        if (p.BR <= 16) {
            float s = 0.f;
            if (r_out < p.BR) {
                const float2 *src = reinterpret_cast<const float2 *>(part + r_out * kPartStride + grp * 16);
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const float2 v = src[q];
                    s += v.x;
                    s += v.y;
                }
            }
            const float s2 = s + __shfl_xor(s, 16);
            rs = s2 + __shfl_xor(s2, 32);
        } else {
            float s = 0.f;
            if (r_out < p.BR) {
                const float2 *src = reinterpret_cast<const float2 *>(part + r_out * kPartStride + grp * 32);
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const float2 v = src[q];
                    s += v.x;
                    s += v.y;
                }
            }
            rs = s + __shfl_xor(s, 32);
        }
        yacc += rs;                                               // the same value in every lane group
        __builtin_amdgcn_wave_barrier();                          // table consumed before the next item refills LDS
        if (cur.c0 + p.seg_blocks >= p.nbc) {                     // last segment of a strip
#pragma unroll
            for (int k = 0; k < kKeep; ++k)
                if (npend == grp + k * ngrp) {
                    ykeep[k] = yacc;
                    rowkeep[k] = cur.srow;
                }
            if constexpr (CELL != 0) ysum = yacc;
            yacc = 0.f;
            ++npend;
        }
        cur = nxt;
    }
    if constexpr (CELL == 0) {
        store_kept();
    } else {
        // The waves' strips are the gate rows of hidden units u0 .. u0 + BR - 1.  Their sums meet in LDS (the x area
        // is free once every wave has multiplied), then one thread per hidden unit applies the cell.  The gate
        // pre-activations (without bias) are stored as the product alone would store them.
        __syncthreads();
        float *gl = reinterpret_cast<float *>(smem);              // [NWV][32]
        if (grp == 0 && r_out < p.BR) gl[wave * 32 + r_out] = ysum;
        __syncthreads();
        if (tid < p.BR) {
            const RnnCell &cl = p.cell;
            const int64_t H = cl.H, j = (int64_t)blockIdx.x * p.BR + tid;
            GRIM_GLOBAL float *y0 = (GRIM_GLOBAL float *)p.y + bq;
            if constexpr (CELL == 1) {
                const float pi = gl[tid], pf = gl[32 + tid], pg = gl[64 + tid], po = gl[96 + tid];
                y0[j * p.ldy] = pi; y0[(H + j) * p.ldy] = pf; y0[(2 * H + j) * p.ldy] = pg; y0[(3 * H + j) * p.ldy] = po;
                float c = cell_st;
                const float h = lstm_cell_apply(pi + cell_b[0], pf + cell_b[1], pg + cell_b[2], po + cell_b[3], c);
                cl.c[j * cl.ldc + bq] = c;
                if (cl.h32) cl.h32[j * cl.ldh32 + bq] = h;
                if (cl.h) rnn_store_h(cl.h, cl.hdt, j * cl.ldh + bq, h);
            } else {
                GRIM_GLOBAL float *y1 = y0 + p.y_stride;
                float pi[3], ph[3];
#pragma unroll
                for (int k = 0; k < 3; ++k) {
                    const float vi = gl[k * 32 + tid], vh = gl[(3 + k) * 32 + tid];
                    y0[(k * H + j) * p.ldy] = vi;
                    y1[(k * H + j) * p.ldy] = vh;
                    pi[k] = vi + cell_b[k];
                    ph[k] = vh + cell_b[3 + k];
                }
                const float h = gru_cell_apply(pi[0], pi[1], pi[2], ph[0], ph[1], ph[2], cell_st);
                cl.c[j * cl.ldc + bq] = h;
                if (cl.h) rnn_store_h(cl.h, cl.hdt, j * cl.ldh + bq, h);
            }
        }
    }
}

template <int DT, int KR, int KC, int KEEP>
static grim_status launch_exact_inst(const GemvParams &p, dim3 grid, size_t lds, hipStream_t stream) {
    auto kern = bcr_spmv_wave_exact<DT, KR, KC, 0, KEEP>;
    static std::atomic<bool> attr_done{false};
    if (lds > 64 * 1024 && !attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) {
            (void)hipGetLastError();
            return GRIM_ERR_DEVICE;
        }
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, stream, p);
    return hipGetLastError() == hipSuccess ? GRIM_OK : GRIM_ERR_DEVICE;
}

template <int DT, int KR, int KC, int CELL>
static grim_status launch_cell_inst(const GemvParams &p, dim3 grid, size_t lds, hipStream_t stream) {
    auto kern = bcr_spmv_wave_exact<DT, KR, KC, CELL>;
    static std::atomic<bool> attr_done{false};
    if (lds > 64 * 1024 && !attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) {
            (void)hipGetLastError();
            return GRIM_ERR_DEVICE;
        }
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(exact_waves(CELL) * 64), lds, stream, p);
    return hipGetLastError() == hipSuccess ? GRIM_OK : GRIM_ERR_DEVICE;
}

// the recurrent-cell variants are compiled for the two-byte element types
template <int DT, int CELL>
static grim_status launch_cell(const GemvParams &p, int kr, int kc, dim3 grid, size_t lds, hipStream_t stream) {
#define GRIM_CELL(R, C)                                                                    \
    if constexpr ((R) * (C) * 2 % 16 == 0 && (R) * (C) * 2 <= 384)                         \
        if (kr == (R) && kc == (C)) return launch_cell_inst<DT, R, C, CELL>(p, grid, lds, stream);
    GRIM_CELL(4, 4) GRIM_CELL(4, 8) GRIM_CELL(4, 12) GRIM_CELL(4, 16)
    GRIM_CELL(8, 4) GRIM_CELL(8, 8) GRIM_CELL(8, 12) GRIM_CELL(8, 16)
    GRIM_CELL(16, 4) GRIM_CELL(16, 8) GRIM_CELL(16, 12)
#undef GRIM_CELL
    return GRIM_ERR_UNSUPPORTED;
}

// Compiled (kept rows, kept columns) pairs; a block must be a whole number of 16-byte vectors
// and at most 24 of them (the block lives in registers).
template <int DT>
static grim_status launch_exact(const GemvParams &p, int kr, int kc, dim3 grid, size_t lds, hipStream_t stream) {
    constexpr int ESZ = (int)sizeof(typename GElem<DT>::type);
#define GRIM_EXACT(R, C)                                                                   \
    if constexpr ((R) * (C) * ESZ % 16 == 0 && (R) * (C) * ESZ <= 384)                     \
        if (kr == (R) && kc == (C))                                                        \
            return p.sps > 8 ? launch_exact_inst<DT, R, C, 8>(p, grid, lds, stream)        \
                             : launch_exact_inst<DT, R, C, 4>(p, grid, lds, stream);
    GRIM_EXACT(4, 4) GRIM_EXACT(4, 8) GRIM_EXACT(4, 12) GRIM_EXACT(4, 16)
    GRIM_EXACT(8, 4) GRIM_EXACT(8, 8) GRIM_EXACT(8, 12) GRIM_EXACT(8, 16)
    GRIM_EXACT(16, 4) GRIM_EXACT(16, 8) GRIM_EXACT(16, 12)
#undef GRIM_EXACT
    return GRIM_ERR_UNSUPPORTED;
}

// ------------------------------------------------------------------------------------------
// 2..8 right-hand sides, every block keeping exactly KR rows and KC columns, strips of at most 64
// column blocks: the uniform wave-per-strip scheme with a loop over the right-hand sides around
// everything after the weights.  A strip's weights are fetched and parked once; for each column
// of x the lane gathers its KC activations, multiplies, and the row sums go through the
// [strip row][block] table.  Results collect in a per-wave LDS tile [right-hand side][strip row]
// and leave with the next strip's first store slot (see the one-column kernel for why a store
// is not issued just before a wait for loads), coalesced when y is contiguous.
// x sits in LDS as [k][right-hand side], shared by the workgroup's waves.
// ------------------------------------------------------------------------------------------
// B8 (eight right-hand sides of 2-byte elements): a row of x is 16 bytes, so a lane takes all eight values of a kept
// column with ONE 16-byte LDS read instead of eight 2-byte ones, and every column block's rows are followed by 16 bytes
// of padding in LDS: the lanes of such a read (one per block) then start 4 banks apart instead of all in the same bank
// (rows of 32 blocks x 16 bytes are 512 bytes apart: 2-byte reads at that stride take 64 turns).
template <int DT, int KR, int KC, bool B8 = false>
__global__ void __launch_bounds__(512) bcr_spmv_wave_exact_b(GemvParams p) {
    using T = typename GElem<DT>::type;
    constexpr int ESZ = (int)sizeof(T);
    static_assert(!B8 || ESZ == 2, "eight 2-byte elements are one 16-byte row");
    constexpr int NV = KR * KC * ESZ / 16;       // 16-byte vectors per block
    constexpr int PB = exact_pad_period(NV);     // one vector of padding after every PB blocks (0: none)
    static_assert(KR * KC * ESZ % 16 == 0 && (ESZ == 4 || KC % 2 == 0) && KC <= 32 && KR <= 32, "block shape");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, nthreads = blockDim.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int B = B8 ? 8 : p.batch;
    const int xbytes = ((p.K * B + (B8 ? p.nbc * 8 : 0)) * ESZ + 15) & ~15;
    T *xs = reinterpret_cast<T *>(smem);
    char *wl = smem + xbytes + wave * p.wbytes;
    float *part = reinterpret_cast<float *>(wl);                  // reuses the weights' space
    float *ybuf = reinterpret_cast<float *>(wl + p.wbytes - 8 * 32 * 4);   // [8][32], behind weights and table

    const int64_t mi = blockIdx.y;
    const GemvGlobal d = to_global(p.table ? p.table[mi] : mi ? p.second : p.single);
    const GRIM_GLOBAL char *W = d.weights;
    const GRIM_GLOBAL T *x = (const GRIM_GLOBAL T *)p.x + mi * p.x_stride;
    GRIM_GLOBAL float *y = (GRIM_GLOBAL float *)p.y + mi * p.y_stride;

    const int64_t t0 = ((int64_t)blockIdx.x * (nthreads >> 6) + wave) * p.sps;
    const int nstrips = p.nbr_total - t0 < p.sps ? (int)(p.nbr_total - t0) : p.sps;   // <= 0: nothing to do
    const int nitems = nstrips > 0 ? nstrips : 0;
    const int nb = p.nbc;                                         // <= 64: one lane per block of the strip
    const int nvec = nb * NV;

    struct Item { unsigned int rm, cm; int srow; };
    gu32x4 wreg[NV];
    auto fetch = [&](int it, Item &I) {
        const int64_t t = t0 + it;
        const int64_t blk0 = t * p.nbc;
        const GRIM_GLOBAL char *src = W + (size_t)blk0 * (NV * 16);
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            int v = lane + i * 64;
            v = v < nvec ? v : nvec - 1;
            wreg[i] = *reinterpret_cast<const GRIM_GLOBAL gu32x4 *>(src + (unsigned int)(v * 16));
        }
        I.rm = 0;
        I.cm = KC == 32 ? 0xffffffffu : (1u << (KC & 31)) - 1u;   // idle lanes: any KC columns, no rows
        if (lane < nb) {
            const gu32x2 mm = *reinterpret_cast<const GRIM_GLOBAL gu32x2 *>(d.masks + 2 * (blk0 + lane));
            I.rm = mm.x;
            I.cm = mm.y;
        }
        I.srow = d.strip_order[t];
    };

    // output lanes: (strip row, lane group); 4 groups of 16 lanes up to 16 strip rows, else 2 of 32
    const int r_out = p.BR <= 16 ? lane & 15 : lane & 31;
    const int grp = p.BR <= 16 ? lane >> 4 : lane >> 5;
    int pend_row = -1;                                            // strip whose sums wait in ybuf
    auto flush = [&]() {
        if (pend_row >= 0) {
            for (int e = lane; e < p.BR * B; e += 64) {
                const int r = e / B, b = e - r * B;
                y[((int64_t)pend_row * p.BR + r) * p.ldy + b] = ybuf[b * 32 + r];
            }
        }
        pend_row = -1;
    };

    Item cur, nxt;
    if (p.xvec16) {
        const int nxv = p.K * B * ESZ / 16;
        const GRIM_GLOBAL gu32x4 *xsrc = reinterpret_cast<const GRIM_GLOBAL gu32x4 *>(x);
        gu32x4 xreg[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int v = tid + i * nthreads;
            v = v < nxv ? v : nxv - 1;
            xreg[i] = xsrc[v];
        }
        if (nitems) fetch(0, cur);
        // (B8: 16-byte unit v is row v of x; one unit of padding behind every block's BC rows)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int v = tid + i * nthreads;
            if (v < nxv) reinterpret_cast<gu32x4 *>(xs)[B8 ? v + v / p.BC : v] = xreg[i];
        }
        for (int v = tid + 4 * nthreads; v < nxv; v += nthreads) reinterpret_cast<gu32x4 *>(xs)[B8 ? v + v / p.BC : v] = xsrc[v];
    } else {
        if (nitems) fetch(0, cur);
        for (int e = tid; e < p.K * B; e += nthreads) {
            const int k = e / B;
            xs[B8 ? e + k / p.BC * 8 : e] = x[(int64_t)k * p.ldx + (e - k * B)];
        }
    }
    __syncthreads();
    if (!nitems) return;
    for (int it = 0; it < nitems; ++it) {
        const unsigned int rm = cur.rm, cm = cur.cm;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int v = lane + i * 64;
            const int slot = PB ? v + v / (NV * PB) : v;
            if (v < nvec) *reinterpret_cast<gu32x4 *>(wl + slot * 16) = wreg[i];
        }
        __builtin_amdgcn_wave_barrier();
        flush();                                                  // the previous strip's sums
        nxt = cur;
        if (it + 1 < nitems) fetch(it + 1, nxt);

        // where this block's KC activations start in x (element index of right-hand side 0)
        int xo[KC];
        {
            int xblk = lane < p.nbc ? lane : p.nbc - 1;
            unsigned int m = cm;
#pragma unroll
            for (int j = 0; j < KC; ++j) {
                const int col = __builtin_ctz(m);                 // KC bits are set
                m &= m - 1;
                xo[j] = (xblk * p.BC + col) * B + (B8 ? xblk * 8 : 0);
            }
        }
        gu32x4 w[NV];
        {
            const gu32x4 *wb = reinterpret_cast<const gu32x4 *>(wl) + lane * NV + (PB ? lane / PB : 0);
#pragma unroll
            for (int j = 0; j < NV; ++j) w[j] = wb[j];
        }
        // The [strip row][block] table takes the place of the parked weights.  It is cleared once per strip: every
        // right-hand side writes the same entries (the rows its block keeps), so the next one overwrites them.
        __builtin_amdgcn_wave_barrier();                          // every lane holds its block in registers
        for (int z = lane; z < (p.BR * kPartStride + 3) / 4; z += 64)
            reinterpret_cast<gu32x4 *>(part)[z] = gu32x4{0u, 0u, 0u, 0u};
        __builtin_amdgcn_wave_barrier();
        gu32x4 xv[B8 ? KC : 1];                                   // B8: the eight values of every kept column
        if constexpr (B8) {
#pragma unroll
            for (int j = 0; j < KC; ++j) xv[j] = *reinterpret_cast<const gu32x4 *>(xs + xo[j]);
        }
        auto column = [&](int b, bool odd, int q) {               // right-hand side b = 2 q + odd (B8: q and odd constants)
            T xe[KC];
            if constexpr (!B8) {
#pragma unroll
                for (int j = 0; j < KC; ++j) xe[j] = xs[xo[j] + b];
            }
            float acc[KR];
            if constexpr (DT == GRIM_F32) {
#pragma unroll
                for (int i = 0; i < KR; ++i) {
                    float a = 0.f;
#pragma unroll
                    for (int j = 0; j < KC; ++j) {
                        const int q = i * KC + j;
                        const unsigned int wd = w[q >> 2][q & 3];
                        a = __builtin_fmaf(__builtin_bit_cast(float, wd), xe[j], a);
                    }
                    acc[i] = a;
                }
            } else {
                unsigned int xp[KC / 2];
#pragma unroll
                for (int h = 0; h < KC / 2; ++h) {
                    if constexpr (B8) {
                        // halves b of two kept columns' dwords q, side by side (low: column 2 h, high: column 2 h + 1)
                        xp[h] = __builtin_amdgcn_perm(xv[2 * h + 1][q], xv[2 * h][q], odd ? 0x07060302u : 0x05040100u);
                    } else {
                        unsigned short lo, hi;
                        __builtin_memcpy(&lo, &xe[2 * h], 2);
                        __builtin_memcpy(&hi, &xe[2 * h + 1], 2);
                        xp[h] = (unsigned int)lo | ((unsigned int)hi << 16);
                    }
                }
#pragma unroll
                for (int i = 0; i < KR; ++i) {
                    float a = 0.f;
#pragma unroll
                    for (int h = 0; h < KC / 2; ++h) {
                        const int qq = i * (KC / 2) + h;
                        const unsigned int wd = w[qq >> 2][qq & 3];
                        if constexpr (DT == GRIM_F16)
                            a = __builtin_amdgcn_fdot2(__builtin_bit_cast(gh2, wd), __builtin_bit_cast(gh2, xp[h]), a, false);
                        else
                            a = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(gb2, wd), __builtin_bit_cast(gb2, xp[h]), a, false);
                    }
                    acc[i] = a;
                }
            }
            if (rm) {
                unsigned int m = rm;
#pragma unroll
                for (int i = 0; i < KR; ++i) {
                    const int r = __builtin_ctz(m);               // KR bits are set
                    m &= m - 1;
                    part[r * kPartStride + lane] = acc[i];
                }
            }
            __builtin_amdgcn_wave_barrier();
            float rs;
            if (p.BR <= 16) {
                float s = 0.f;
                if (r_out < p.BR) {
                    const float2 *src = reinterpret_cast<const float2 *>(part + r_out * kPartStride + grp * 16);
#pragma unroll
                    for (int q = 0; q < 8; ++q) {
                        const float2 v = src[q];
                        s += v.x;
                        s += v.y;
                    }
                }
                const float s2 = s + __shfl_xor(s, 16);
                rs = s2 + __shfl_xor(s2, 32);
            } else {
                float s = 0.f;
                if (r_out < p.BR) {
                    const float2 *src = reinterpret_cast<const float2 *>(part + r_out * kPartStride + grp * 32);
#pragma unroll
                    for (int q = 0; q < 16; ++q) {
                        const float2 v = src[q];
                        s += v.x;
                        s += v.y;
                    }
                }
                rs = s + __shfl_xor(s, 32);
            }
            if (grp == 0 && r_out < p.BR) ybuf[b * 32 + r_out] = rs;
            __builtin_amdgcn_wave_barrier();                      // table consumed before the next right-hand side writes it
        };
        if constexpr (B8) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                column(2 * q, false, q);
                column(2 * q + 1, true, q);
            }
        } else {
            for (int b = 0; b < B; ++b) column(b, false, 0);
        }
        pend_row = cur.srow;
        cur = nxt;
    }
    flush();
}

// kept elements per block up to which the eight-column form (all of x's values of a block in registers) fits the
// register file without spills
constexpr int kExactB8MaxBlock = 96;

template <int DT, int KR, int KC, bool B8>
static grim_status launch_exact_b_inst(const GemvParams &p, dim3 grid, int threads, size_t lds, hipStream_t stream) {
    auto kern = bcr_spmv_wave_exact_b<DT, KR, KC, B8>;
    static std::atomic<bool> attr_done{false};
    if (lds > 64 * 1024 && !attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) {
            (void)hipGetLastError();
            return GRIM_ERR_DEVICE;
        }
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(threads), lds, stream, p);
    return hipGetLastError() == hipSuccess ? GRIM_OK : GRIM_ERR_DEVICE;
}

template <int DT>
static grim_status launch_exact_b(const GemvParams &p, int kr, int kc, dim3 grid, int threads, size_t lds, hipStream_t stream) {
    constexpr int ESZ = (int)sizeof(typename GElem<DT>::type);
#define GRIM_EXACT(R, C)                                                                   \
    if constexpr ((R) * (C) * ESZ % 16 == 0 && (R) * (C) * ESZ <= 384)                     \
        if (kr == (R) && kc == (C)) {                                                      \
            if constexpr ((R) * (C) <= kExactB8MaxBlock)                                       \
                if (p.batch == 8) return launch_exact_b_inst<DT, R, C, true>(p, grid, threads, lds, stream); \
            return launch_exact_b_inst<DT, R, C, false>(p, grid, threads, lds, stream);        \
        }
    GRIM_EXACT(4, 4) GRIM_EXACT(4, 8) GRIM_EXACT(4, 12) GRIM_EXACT(4, 16)
    GRIM_EXACT(8, 4) GRIM_EXACT(8, 8) GRIM_EXACT(8, 12) GRIM_EXACT(8, 16)
    GRIM_EXACT(16, 4) GRIM_EXACT(16, 8) GRIM_EXACT(16, 12)
#undef GRIM_EXACT
    return GRIM_ERR_UNSUPPORTED;
}

template <int DT, int B>
static grim_status launch_vec(const GemvParams &p, int vec, dim3 grid, size_t lds, hipStream_t stream) {
#define GRIM_GEMV(V)                                                                                          \
    {                                                                                                         \
        auto kern = bcr_spmv<DT, B, V>;                                                                       \
        static std::atomic<bool> attr_done{false};                                                                        \
        if (lds > 64 * 1024 && !attr_done) {                                                                  \
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) { \
                (void)hipGetLastError();                                                                      \
                return GRIM_ERR_DEVICE;                                                                       \
            }                                                                                                 \
            attr_done = true;                                                                                 \
        }                                                                                                     \
        hipLaunchKernelGGL(kern, grid, dim3(gemv_threads(B)), lds, stream, p);                                \
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

// Strips a wave of the wave-per-strip kernels walks: 1 when the launch is small, up to max_sps
// while at least 512 workgroups (two per compute unit) remain -- a large launch then is one round of
// long-lived workgroups.
static int spmv_compute_units();

static int wave_strips_per_wave(int64_t count, int64_t nbr, int max_sps) {
    int sps = 1;
    while (sps < max_sps && count * ((nbr + 4 * sps * 2 - 1) / (4 * sps * 2)) >= 512) sps *= 2;
    return sps;
}

grim_status launch_spmv(const GemvDesc *table, const GemvDesc &single, const GemvDesc *second, int32_t count, int64_t M, int64_t K, int32_t BR,
                        int32_t BC, int32_t dtype, int32_t ukr, int32_t ukc, int32_t vec, int32_t krmax, int32_t kcmax,
                        const void *x, int64_t x_stride, int32_t batch, int64_t ldx, float *y, int64_t y_stride, int64_t ldy,
                        hipStream_t stream) {
    if (BR > 32 || BC > 32 || batch < 1 || batch > 8) return GRIM_ERR_UNSUPPORTED;
    const int esz = dtype_size(dtype);
    const int64_t nbr = M / BR;
    if (nbr > 0x7fffffff || count > 65535) return GRIM_ERR_SHAPE;
    if (!table && count != (second ? 2 : 1)) return GRIM_ERR_SHAPE;
    if (krmax < 1) krmax = 1;
    if (kcmax < 1) kcmax = 1;
    GemvParams p;
    p.table = table;
    p.single = single;
    p.second = second ? *second : single;
    p.BR = BR; p.BC = BC; p.nbc = (int32_t)(K / BC); p.K = (int32_t)K;
    p.nbr_total = (int32_t)nbr;
    p.sps = 1;
    p.wpg = 4;
    p.batch = batch;
    p.ukr = ukr; p.ukc = ukc;
    p.krmax = krmax;
    p.kcmax = kcmax;
    int lpb = 4;
    while (lpb < krmax && lpb < 32) lpb <<= 1;
    if (krmax <= 8 && krmax > 4) lpb = 8;
    p.lpb_shift = lpb == 4 ? 2 : lpb == 8 ? 3 : lpb == 16 ? 4 : 5;
    // a segment's weights (plus the 16-byte alignment window) must fit the per-thread fetch budget
    const int64_t blk_bytes = (int64_t)krmax * kcmax * esz;
    int64_t seg = (kGemvWBytes - 32) / blk_bytes;
    if (seg < 1) return GRIM_ERR_UNSUPPORTED;
    if (seg > kSegMax) seg = kSegMax;
    p.seg_blocks = (int32_t)seg;
    p.wbytes = (int32_t)((seg * blk_bytes + 32 + 15) & ~int64_t(15));
    p.x = x; p.y = y; p.x_stride = x_stride; p.y_stride = y_stride; p.ldx = ldx; p.ldy = ldy;
    const bool contiguous = ldx == batch && reinterpret_cast<uintptr_t>(x) % 16 == 0 &&
                            (K * batch * esz) % 16 == 0 && (count == 1 || (x_stride * esz) % 16 == 0);
    p.xvec16 = contiguous ? 1 : 0;
    // several columns as sets of workgroups of the one-column kernel, while all sets run in one round
    const bool column_sets = batch > 1 && spmv_column_sets_ok(count, nbr, batch);
    if ((batch == 1 || column_sets) && (int64_t)K * esz <= 32 * 1024) {
        // uniformly pruned matrix: one wave per strip, one lane per block
        if (ukr > 0 && ukc > 0 && (ukr * ukc * esz) % 16 == 0 && ukr * ukc * esz <= 384) {
            const int nv = ukr * ukc * esz / 16;
            GemvParams q = p;
            q.seg_blocks = 64;
            int64_t wb = (int64_t)exact_region_vectors(nv) * 16;
            const int64_t table = ((int64_t)BR * kPartStride * 4 + 15) & ~int64_t(15);
            if (wb < table) wb = table;
            q.wbytes = (int32_t)wb;
            const size_t wlds = ((((size_t)K + (size_t)(K / BC) * exact_x_skew(BC, esz)) * esz + 15) & ~size_t(15)) + 4 * (size_t)wb;
            q.sps = batch == 1 ? wave_strips_per_wave(count, nbr, 16) : 1;
            if (batch > 1) q.xvec16 = 0;                        // a column of x is strided
            // while a workgroup per strip (or per two) still leaves every workgroup a compute unit of its own, take it
            const int64_t cus = spmv_compute_units(), strips = (int64_t)count * nbr * batch;
            q.wpg = q.sps == 1 && strips <= cus ? 1 : q.sps == 1 && strips <= 2 * cus ? 2 : 4;
            dim3 wgrid((unsigned)((nbr + q.wpg * q.sps - 1) / (q.wpg * q.sps)), (unsigned)count, (unsigned)batch);
            grim_status st = GRIM_ERR_UNSUPPORTED;
            if (wlds <= 160 * 1024) {
                switch (dtype) {
                    case GRIM_F32: st = launch_exact<GRIM_F32>(q, ukr, ukc, wgrid, wlds, stream); break;
                    case GRIM_F16: st = launch_exact<GRIM_F16>(q, ukr, ukc, wgrid, wlds, stream); break;
                    case GRIM_BF16: st = launch_exact<GRIM_BF16>(q, ukr, ukc, wgrid, wlds, stream); break;
                }
            }
            if (st != GRIM_ERR_UNSUPPORTED) return st;
        }
    }
    if (batch > 1 && dtype != GRIM_F32 && ukr > 0 && ukc > 0 && (ukr * ukc * esz) % 16 == 0 && ukr * ukc * esz <= 384 &&
        K / BC <= 64 && (int64_t)K * batch * esz <= 64 * 1024 && (int64_t)count * nbr >= 1024) {
        // uniform blocks, several right-hand sides, a launch of at least 128 workgroups: wave per
        // strip, 8 waves share x in LDS (smaller launches are quicker with a workgroup per strip)
        const int nv = ukr * ukc * esz / 16, nw = 8;
        GemvParams q = p;
        q.seg_blocks = 64;
        int64_t wb = (int64_t)exact_region_vectors(nv) * 16;
        const int64_t table = ((int64_t)BR * kPartStride * 4 + 15) & ~int64_t(15);
        if (wb < table) wb = table;
        wb += 8 * 32 * 4;                                       // the wave's result tile
        q.wbytes = (int32_t)wb;
        // (eight right-hand sides: 16 bytes of padding behind every column block's rows of x)
        const bool b8 = batch == 8 && ukr * ukc <= kExactB8MaxBlock;
        const size_t wlds = ((((size_t)K * batch + (b8 ? (size_t)(K / BC) * 8 : 0)) * esz + 15) & ~size_t(15)) + nw * (size_t)wb;
        int sps = 1;
        while (sps < 4 && (int64_t)count * ((nbr + nw * sps * 2 - 1) / (nw * sps * 2)) >= 512) sps *= 2;
        q.sps = sps;
        dim3 wgrid((unsigned)((nbr + nw * sps - 1) / (nw * sps)), (unsigned)count);
        grim_status st = GRIM_ERR_UNSUPPORTED;
        if (wlds <= 160 * 1024)
            st = dtype == GRIM_F16 ? launch_exact_b<GRIM_F16>(q, ukr, ukc, wgrid, nw * 64, wlds, stream)
                                   : launch_exact_b<GRIM_BF16>(q, ukr, ukc, wgrid, nw * 64, wlds, stream);
        if (st != GRIM_ERR_UNSUPPORTED) return st;
    }
    const int rb = BR * batch;
    const int nseg = gemv_threads(batch) / rb;
    const size_t lds = (size_t)p.wbytes + 16 + 2 * kSegMax * 4 + (kSegMax + 4) * 4 +
                       (((size_t)seg * gemv_xg_stride(kcmax, batch) * esz + 15) & ~size_t(15)) +
                       (size_t)((seg * krmax * batch + 4) & ~3) * 4 + (size_t)((nseg * rb + 3) & ~3) * 4 +
                       (((size_t)K * batch * esz + 15) & ~size_t(15));
    if (lds > 160 * 1024) return GRIM_ERR_UNSUPPORTED;
    dim3 grid((unsigned)nbr, (unsigned)count);
    switch (dtype) {
        case GRIM_F32: return launch_batch<GRIM_F32>(p, batch, vec, grid, lds, stream);
        case GRIM_F16: return launch_batch<GRIM_F16>(p, batch, vec, grid, lds, stream);
        case GRIM_BF16: return launch_batch<GRIM_BF16>(p, batch, vec, grid, lds, stream);
    }
    return GRIM_ERR_DTYPE;
}

bool spmv_cell_applies(int kind, int64_t M, int64_t K, int32_t BR, int32_t BC, int32_t dtype, int32_t ukr, int32_t ukc, int64_t H) {
    const int gates = kind == 1 ? 4 : 3, esz = 2;
    if (kind != 1 && kind != 2) return false;
    if (BR > 32 || BC > 32 || dtype == GRIM_F32 || ukr <= 0 || ukc <= 0) return false;
    if (H < 1 || H > 0x7fffffff || M != (int64_t)gates * H || H % BR != 0 || K % BC != 0) return false;
    if ((ukr * ukc * esz) % 16 != 0 || ukr * ukc * esz > 384 || K * esz > 32 * 1024) return false;
    if (!((ukr == 4 || ukr == 8 || ukr == 16) && (ukc == 4 || ukc == 8 || ukc == 12 || ukc == 16)) || (ukr == 16 && ukc == 16))
        return false;                                              // the pairs launch_cell is compiled for
    const int nv = ukr * ukc * esz / 16;
    int64_t wb = (int64_t)exact_region_vectors(nv) * 16;
    const int64_t table = ((int64_t)BR * kPartStride * 4 + 15) & ~int64_t(15);
    if (wb < table) wb = table;
    const int64_t lds = (kind == 2 ? 2 : 1) * (((K + K / BC * exact_x_skew(BC, esz)) * esz + 15) & ~int64_t(15)) + exact_waves(kind) * wb;
    return lds <= 160 * 1024;
}

// One recurrent step in one launch: the gate product(s) with the cell in the epilogue (kind 1: LSTM, one matrix of 4H
// rows; kind 2: GRU, two matrices of 3H rows with the same K, block size and kept counts).  One right-hand side,
// fp16 / bf16, every block keeping the same kr x kc, H a multiple of BR.  GRIM_ERR_UNSUPPORTED when the matrices do not
// qualify: the caller then runs the product(s) and the cell as separate launches.
static int spmv_compute_units() {
    static std::atomic<int> cached{0};
    int n = cached.load();
    if (n > 0) return n;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) {
        (void)hipGetLastError();
        return 0;
    }
    cached = n;
    return n;
}

// the (kept rows, kept columns) pairs the one-column wave-per-strip kernel is compiled for
bool spmv_exact_applies(int32_t dtype, int32_t ukr, int32_t ukc, int64_t K) {
    const int esz = dtype_size(dtype);
    if (!((ukr == 4 || ukr == 8 || ukr == 16) && (ukc == 4 || ukc == 8 || ukc == 12 || ukc == 16))) return false;
    return (ukr * ukc * esz) % 16 == 0 && ukr * ukc * esz <= 384 && K * esz <= 32 * 1024;
}

// `count` products of nbr strips each on `batch` columns as sets of workgroups of the one-column kernel (four strips per
// workgroup): do all sets fit the GPU in one round?
bool spmv_column_sets_ok(int64_t count, int64_t nbr, int32_t batch) {
    return batch >= 1 && batch <= 8 && count * ((nbr + 3) / 4) * batch <= spmv_compute_units();
}

// A set of H / BR workgroups per column of x pays while all sets run at once, one workgroup per compute unit (a GRU
// layer of 1024 hidden units: 6.0 us with 1 column, 6.9 us with 8; with 32 columns, four rounds of workgroups, 22.9 us
// against 8.4 us for the products on the matrix cores followed by the cell kernel).
bool spmv_cell_batch_ok(int64_t H, int32_t BR, int32_t batch) {
    if (batch < 1 || batch > kCellMaxBatch || BR < 1) return false;
    if (batch == 1) return true;
    return H / BR * batch <= spmv_compute_units();
}

grim_status launch_spmv_cell(int kind, const GemvDesc &d1, const GemvDesc *d2, int64_t M, int64_t K, int32_t BR, int32_t BC,
                             int32_t dtype, int32_t ukr, int32_t ukc, const void *x, int64_t x_stride, int32_t batch, int64_t ldx,
                             float *y, int64_t y_stride, int64_t ldy, const RnnCell &cell, hipStream_t stream) {
    if ((kind == 2 && !d2) || !spmv_cell_applies(kind, M, K, BR, BC, dtype, ukr, ukc, cell.H)) return GRIM_ERR_UNSUPPORTED;
    if (!spmv_cell_batch_ok(cell.H, BR, batch)) return GRIM_ERR_UNSUPPORTED;
    const int esz = 2;
    const int64_t groups = cell.H / BR;
    if (groups > 0x7fffffff) return GRIM_ERR_SHAPE;
    GemvParams p;
    p.table = nullptr;
    p.single = d1;
    p.second = d2 ? *d2 : d1;
    p.BR = BR; p.BC = BC; p.nbc = (int32_t)(K / BC); p.K = (int32_t)K;
    p.nbr_total = (int32_t)(M / BR);
    p.sps = 1;
    p.wpg = 4;
    p.batch = 1;
    p.ukr = ukr; p.ukc = ukc; p.krmax = ukr; p.kcmax = ukc; p.lpb_shift = 2;
    p.seg_blocks = 64;
    const int nv = ukr * ukc * esz / 16;
    int64_t wb = (int64_t)exact_region_vectors(nv) * 16;
    const int64_t table = ((int64_t)BR * kPartStride * 4 + 15) & ~int64_t(15);
    if (wb < table) wb = table;
    p.wbytes = (int32_t)wb;
    p.x = x; p.y = y; p.x_stride = x_stride; p.y_stride = y_stride; p.ldx = ldx; p.ldy = ldy;
    p.xvec16 = (ldx == 1 && reinterpret_cast<uintptr_t>(x) % 16 == 0 && (K * esz) % 16 == 0 &&
                (kind == 1 || (x_stride * esz) % 16 == 0)) ? 1 : 0;
    p.cell = cell;
    const int nvecs = kind == 2 ? 2 : 1, nw = exact_waves(kind);
    const size_t lds = nvecs * ((((size_t)K + (size_t)(K / BC) * exact_x_skew(BC, esz)) * esz + 15) & ~size_t(15)) + nw * (size_t)wb;
    if (lds > 160 * 1024) return GRIM_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)groups, (unsigned)batch);
    if (kind == 1)
        return dtype == GRIM_F16 ? launch_cell<GRIM_F16, 1>(p, ukr, ukc, grid, lds, stream)
                                 : launch_cell<GRIM_BF16, 1>(p, ukr, ukc, grid, lds, stream);
    return dtype == GRIM_F16 ? launch_cell<GRIM_F16, 2>(p, ukr, ukc, grid, lds, stream)
                             : launch_cell<GRIM_BF16, 2>(p, ukr, ukc, grid, lds, stream);
}

}  // namespace grim

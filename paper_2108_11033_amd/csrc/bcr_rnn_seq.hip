// A recurrent layer over a whole sequence in ONE launch (Section 3.1: an RNN layer is one matrix-vector product per
// time step; Section 6.3 times the GRU step by step, where every step pays a kernel launch and re-reads the weights).
//
// Up to 32 independent sequences run side by side (a batch).  A recurrent layer of 1024 hidden units occupies 32 of the
// 256 compute units, so the sequences are first spread over further sets of workgroups (grid.y: each set holds its
// own copy of the weights in registers and exchanges h only within itself, at the pace of a single sequence); when the
// compute units are used up a workgroup carries several sequences in turn on one set of weights.
// A workgroup owns BR hidden units for the whole sequence.  Its waves take the strips that hold these units' gate
// rows (LSTM: 4 strips of [W_ih | W_hh]; GRU: 3 strips of W_i and 3 of W_h), and every lane keeps ONE compact block of
// its strip in registers from the first step to the last: the weights are read from memory once per sequence, not
// once per step.  Per step a workgroup
//   1. parks x_t and h_{t-1} in LDS,
//   2. multiplies (a lane: its block times the block's kept columns of the vector; row sums through a
//      [strip row][block] table in a fixed order, exactly as the one-step kernel does),
//   3. applies the cell to its BR units and publishes their new h.
// Workgroups exchange h through a small buffer of 8-byte words (the new h of one hidden unit for two sequences of the
// batch, already rounded to the element type the next product reads; step tag), two slots used in turn:
// a producer writes a word with one atomic store, consumers re-read a word until its tag is the step they need.
// Values and tag travel together, so no fence and no separate counter is needed.  Slot t & 1 can be overwritten with
// h_{t+2} only by a workgroup that has read all of h_{t+1}, which exists only when every workgroup has finished
// reading h_t: two slots are enough.  Every wait is bounded: after `max_polls` unsuccessful reads a workgroup gives
// up, marks its own words as poisoned (which ends every other workgroup's wait at once) and sets *status; all
// workgroups then leave the kernel normally.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <mutex>

#include "bcr_matrix.hpp"
#include "spmv_common.hpp"

namespace grim {

constexpr unsigned int kSeqPoison = 0xffffffffu;   // tag of a word whose producer has given up
constexpr unsigned int kSeqDefaultPolls = 1u << 21;
constexpr size_t kSeqMaxLds = 160 * 1024 - 256;    // dynamic part: the kernel also has a few static bytes

struct SeqParams {
    GemvDesc d1, d2;               // LSTM: the gate matrix; GRU: W_i and W_h
    const int32_t *pos1, *pos2;    // stored position of every original strip
    int32_t BR, BC;
    int32_t nbc1, nbc2;            // column blocks per strip (<= 64 each)
    int32_t K1, K2;                // LSTM: K1 = I + H; GRU: K1 = I, K2 = H
    int32_t I, H, T;
    int32_t B;                     // sequences side by side (1 .. 32), dealt to grid.y sets of workgroups
    int32_t SPB, NQ;               // sequences per workgroup; pairs of them = exchange words per hidden unit
    int32_t xvec16;                // rows of xs can be copied with 16-byte loads
    const void *xs;                // T x B rows of I inputs, row t * B + b
    int64_t ldxs;
    const void *h0;                // B x H elements: h before the first step
    const float *bias, *bias2;     // LSTM: 4H; GRU: 3H input side, 3H hidden side; null = none
    float *state;                  // LSTM: c, GRU: h in fp32; B x H values, read at the start, written at the end
    void *hs;                      // T x B rows of H outputs in the matrices' element type
    int64_t ldhs;
    float *hs32;                   // optional fp32 copy of the outputs
    int64_t ldhs32;
    unsigned long long *exch;      // grid.y x 2 x NQ x H words (two 16-bit values, tag); all tags zero at launch
    int32_t *status;               // set to 1 by a workgroup that gives up
    uint32_t max_polls;
};

// the bits of v rounded to the element type (nearest even)
template <int DT> __device__ __forceinline__ unsigned short seq_round(float v);
template <> __device__ __forceinline__ unsigned short seq_round<GRIM_F16>(float v) {
    const _Float16 h = (_Float16)v;
    return __builtin_bit_cast(unsigned short, h);
}
template <> __device__ __forceinline__ unsigned short seq_round<GRIM_BF16>(float v) { return rnn_f32_to_bf16(v); }

constexpr int kSeqXVec = 4;   // 16-byte pieces of a step's inputs a thread fetches ahead
constexpr int kSeqPolls = 2;    // reads of an exchange word a waiting workgroup sends out at once ...
constexpr int kSeqPollGap = 8;  // ... this many times 64 cycles apart (2 x 8, 3 x 5 .. 12, 4 x 4 measured: LSTM alike, the GRU best with two)

// MULTI: a workgroup carries more than one sequence
template <int DT, int KR, int KC, int CELL, bool MULTI>
__global__ void __launch_bounds__(exact_waves(CELL) * 64) bcr_rnn_seq(SeqParams p) {
    using T = typename GElem<DT>::type;
    static_assert(sizeof(T) == 2, "two-byte element types");
    constexpr int NWV = exact_waves(CELL), NTHR = NWV * 64;
    constexpr int NV = KR * KC * 2 / 16;
    static_assert(KR * KC * 2 % 16 == 0 && KC % 2 == 0 && KC <= 32 && KR <= 32, "block shape");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int mi = CELL == 2 ? wave / 3 : 0;
    const int gate = CELL == 2 ? wave % 3 : wave;
    const int H = p.H;
    // this workgroup's sequences: b0 .. b0 + B - 1 of the p.B
    const int set = blockIdx.y, b0 = set * p.SPB;
    const int B = MULTI ? (p.SPB < p.B - b0 ? p.SPB : p.B - b0) : 1;
    const int NQ = MULTI ? p.NQ : 1;
    unsigned long long *const exch = p.exch + (size_t)set * 2 * NQ * H;

    // LDS: the B input vectors (x; LSTM: h follows at element I; GRU: the B vectors h after all x) | a
    // [strip row][block] table per wave | the waves' row sums per sequence
    const int xbytes1 = (B * p.K1 * 2 + 15) & ~15;
    const int xbytes = CELL == 2 ? xbytes1 + ((B * p.K2 * 2 + 15) & ~15) : xbytes1;
    const int tbytes = (p.BR * kPartStride * 4 + 15) & ~15;
    T *xin = reinterpret_cast<T *>(smem);
    unsigned short *hin = reinterpret_cast<unsigned short *>(CELL == 2 ? smem + xbytes1 : smem + p.I * 2);
    const int hld = CELL == 2 ? p.K2 : p.K1;                                  // elements from one sequence's h to the next's
    float *part = reinterpret_cast<float *>(smem + xbytes + wave * tbytes);
    float *gl = reinterpret_cast<float *>(smem + xbytes + NWV * tbytes);      // [B][NWV][32]
    __shared__ int flag_word;
    volatile int *flag = &flag_word;

    // this lane's block: weights into registers for the whole sequence
    const GemvGlobal d = to_global(mi ? p.d2 : p.d1);
    const int nbc = mi ? p.nbc2 : p.nbc1;
    const int32_t *pos = mi ? p.pos2 : p.pos1;
    const int64_t t0 = pos[gate * (H / p.BR) + (int)blockIdx.x];
    const int blk_l = lane < nbc ? lane : nbc - 1;                            // idle lanes re-read the last block
    const int64_t blk = t0 * nbc + blk_l;
    gu32x4 w[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j)
        w[j] = *reinterpret_cast<const GRIM_GLOBAL gu32x4 *>(d.weights + (size_t)blk * (NV * 16) + j * 16);
    unsigned int rm = 0, cm = KC == 32 ? 0xffffffffu : (1u << (KC & 31)) - 1u;   // idle lanes: any KC columns, no rows
    if (lane < nbc) {
        const gu32x2 mm = *reinterpret_cast<const GRIM_GLOBAL gu32x2 *>(d.masks + 2 * blk);
        rm = mm.x;
        cm = mm.y;
    }
    const T *xb = ((CELL == 2 && mi) ? reinterpret_cast<const T *>(hin) : xin) + blk_l * p.BC;
    const int xld = (CELL == 2 && mi) ? p.K2 : p.K1;                          // elements from one sequence's vector to the next's

    // the cell's threads: one per (hidden unit, pair of sequences), states and biases in registers
    const int cq = MULTI ? tid / p.BR : 0, cu = tid - cq * p.BR;
    const bool cell_thread = MULTI ? cq < NQ : tid < p.BR;
    const int64_t ju = (int64_t)blockIdx.x * p.BR + cu;
    float st[2] = {0.f, 0.f}, b[6] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (cell_thread) {
#pragma unroll
        for (int k = 0; k < 2; ++k)
            if (2 * cq + k < B) st[k] = p.state[(int64_t)(b0 + 2 * cq + k) * H + ju];
#pragma unroll
        for (int k = 0; k < (CELL == 1 ? 4 : 3); ++k) {
            if (p.bias) b[k] = p.bias[k * (int64_t)H + ju];
            if (CELL == 2 && p.bias2) b[3 + k] = p.bias2[k * (int64_t)H + ju];
        }
    }
    if (tid == 0) *flag = 0;

    const int ngrp = p.BR <= 16 ? 4 : 2;
    const int r_out = p.BR <= 16 ? lane & 15 : lane & 31;
    const int grp = p.BR <= 16 ? lane >> 4 : lane >> 5;
    (void)ngrp;
    const GRIM_GLOBAL unsigned short *h0 = (const GRIM_GLOBAL unsigned short *)p.h0 + (int64_t)b0 * H;
    const GRIM_GLOBAL T *xs0 = (const GRIM_GLOBAL T *)p.xs + (int64_t)b0 * p.ldxs;
    // 16-byte path: the B rows of a step are at most XV pieces per thread, fetched a step ahead
    constexpr int XV = MULTI ? kSeqXVec : 1;
    const int nxv1 = p.I / 8, nxv = B * nxv1;
    gu32x4 xr[XV];
    int64_t xsrc[XV];                  // piece -> element offset inside the step's rows of xs
    int xdst[XV];                      // piece -> element offset in LDS
#pragma unroll
    for (int k = 0; k < XV; ++k) {
        const int v = tid + k * NTHR < nxv ? tid + k * NTHR : 0;
        const int vb = v / nxv1, vi = v - vb * nxv1;
        xsrc[k] = vb * p.ldxs + vi * 8;
        xdst[k] = vb * p.K1 + vi * 8;
        xr[k] = gu32x4{0u, 0u, 0u, 0u};
        if (p.xvec16 && k * NTHR < nxv) xr[k] = *reinterpret_cast<const GRIM_GLOBAL gu32x4 *>(xs0 + xsrc[k]);
    }
    // positions of the block's kept columns, and the [strip row][block] table zeroed once: a lane only ever
    // writes the entries of its block's kept rows, all others stay zero
    unsigned short coff[KC];
    {
        unsigned int m = cm;
#pragma unroll
        for (int j = 0; j < KC; ++j) {
            coff[j] = (unsigned short)__builtin_ctz(m);                 // KC bits are set
            m &= m - 1;
        }
    }
    for (int z = lane; z < (p.BR * kPartStride + 3) / 4; z += 64)
        reinterpret_cast<gu32x4 *>(part)[z] = gu32x4{0u, 0u, 0u, 0u};
    bool gave_up = false;
    __syncthreads();

    for (int t = 0; t < p.T; ++t) {
        // ---- 1. x_t and h_t (the state BEFORE this step: h0, or what step t - 1 published under tag t)
        if (p.xvec16) {
            // x_t was asked for a step ago; x_{t+1} is asked for now and travels while this step waits for h
            const int tn = t + 1 < p.T ? t + 1 : t;
            const GRIM_GLOBAL T *xg = xs0 + (int64_t)tn * p.B * p.ldxs;
#pragma unroll
            for (int k = 0; k < XV; ++k)
                if (k * NTHR < nxv) {                                 // the same for all threads
                    if (tid + k * NTHR < nxv) *reinterpret_cast<gu32x4 *>(xin + xdst[k]) = xr[k];
                    xr[k] = *reinterpret_cast<const GRIM_GLOBAL gu32x4 *>(xg + xsrc[k]);
                }
        } else {
            for (int bb = 0; bb < B; ++bb) {
                const GRIM_GLOBAL T *xg = xs0 + ((int64_t)t * p.B + bb) * p.ldxs;
                for (int e = tid; e < p.I; e += NTHR) xin[bb * p.K1 + e] = xg[e];
            }
        }
        if (t == 0) {
            for (int bb = 0; bb < B; ++bb)
                for (int e = tid; e < H; e += NTHR) hin[bb * hld + e] = h0[(int64_t)bb * H + e];
        } else {
            // Words of two pairs of sequences per round.  A read of an exchange word takes a round trip through the
            // fabric (1.2 us), and the words of step t become visible a little after this workgroup has published
            // its own: read once at a time, the first read comes back too early and the second costs a whole further
            // round trip.  So the first NP reads of every word go out together, a fraction of a round trip apart
            // (loads return in order; every read is issued whether its element exists or not, so that the wait for
            // the oldest leaves the younger ones in flight).
            const unsigned long long *ex = exch + (size_t)(t & 1) * NQ * H;
            constexpr int NJ = MULTI ? 2 : 1;
            constexpr int NP = MULTI ? 2 : kSeqPolls;               // (several sequences: twice the words per read, fewer registers left)
            bool bad = false;
            for (int q0 = 0; q0 < NQ && !bad; q0 += NJ) {
                for (int base = tid; base < H && !bad; base += 4 * NTHR) {
                    unsigned long long v[NJ * 4], w[NP][NJ * 4];
                    auto ask = [&](unsigned long long (&r)[NJ * 4]) {
#pragma unroll
                        for (int j = 0; j < NJ; ++j) {
                            const int q = q0 + j < NQ ? q0 + j : NQ - 1;
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const int e = base + i * NTHR < H ? base + i * NTHR : H - 1;
                                r[j * 4 + i] = __hip_atomic_load(ex + (size_t)q * H + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            }
                        }
                    };
                    // 1: all tags are t, 0: not yet, -1: a workgroup has given up
                    auto seen = [&](const unsigned long long (&r)[NJ * 4]) {
                        int ok = 1;
#pragma unroll
                        for (int k = 0; k < NJ * 4; ++k) {
                            const unsigned int tag = (unsigned int)(r[k] >> 32);
                            if (tag != (unsigned int)t) ok = ok < 0 ? ok : 0;
                            if (tag == kSeqPoison) ok = -1;
                        }
                        return ok;
                    };
                    // NP reads of every word go out at once, a fraction of a round trip apart, and are examined in turn
                    // (straight-line code, so that the wait for an older read leaves the younger ones in flight); a
                    // wave moves on as a whole, each lane with the first complete set of words it has seen (a slot is
                    // written again two steps later at the earliest, so a later read cannot show anything else).
#pragma unroll
                    for (int d = 0; d < NP; ++d) {
                        ask(w[d]);
                        if (d + 1 < NP) __builtin_amdgcn_s_sleep(kSeqPollGap);
                    }
                    unsigned int polls = 0;
                    bool ok = false, dead = false, waiting = true;
#pragma unroll
                    for (int d = 0; d < NP; ++d) {
                        if (waiting) {                              // (the same for the whole wave)
                            const int st_ = seen(w[d]);
                            if (st_ > 0 && !ok) {
#pragma unroll
                                for (int k = 0; k < NJ * 4; ++k) v[k] = w[d][k];
                                ok = true;
                            }
                            dead = dead || st_ < 0 || (!ok && ++polls >= p.max_polls);
                            waiting = __builtin_amdgcn_ballot_w64(!ok && !dead) != 0;
                        }
                    }
                    // not there yet: one read at a time from here on
                    while (!ok && !dead) {
                        __builtin_amdgcn_s_sleep(1);
                        ask(w[0]);
                        const int st_ = seen(w[0]);
                        if (st_ > 0) {
#pragma unroll
                            for (int k = 0; k < NJ * 4; ++k) v[k] = w[0][k];
                            ok = true;
                        }
                        dead = st_ < 0 || (!ok && ++polls >= p.max_polls);
                    }
                    if (!ok) {
                        *flag = 1;
                        bad = true;
                        break;
                    }
#pragma unroll
                    for (int j = 0; j < NJ; ++j) {
                        if (q0 + j < NQ) {
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const int e = base + i * NTHR;
                                if (e < H) {
                                    const unsigned int pair = (unsigned int)v[j * 4 + i];
                                    hin[(2 * (q0 + j)) * hld + e] = (unsigned short)(pair & 0xffffu);
                                    if (2 * (q0 + j) + 1 < B) hin[(2 * (q0 + j) + 1) * hld + e] = (unsigned short)(pair >> 16);
                                }
                            }
                        }
                    }
                }
            }
        }
        __syncthreads();
        if (*flag) {                                                  // the same value for every thread
            gave_up = true;
            break;
        }

        // ---- 2. per sequence: the block's KC activations, the products, the strip's row sums.  One table per wave
        // serves the sequences in turn: a wave's LDS accesses are carried out in order, so the table of the next
        // sequence can be written while the sums of this one are still on their way.  Blocks small enough for the
        // registers take two sequences per pass: the two chains of gather -> products -> table -> sums overlap.
        constexpr int NS = MULTI && KR * KC <= 96 ? 2 : 1;
        auto products = [&](int bb, float (&acc)[KR]) {
            const T *xbb = xb + bb * xld;
            T xe[KC];
#pragma unroll
            for (int j = 0; j < KC; ++j) xe[j] = xbb[coff[j]];
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
        };
        // the lane's sums into the table, then the table entries this lane adds up (16 blocks per quarter of the wave
        // up to 16 strip rows, 32 per half above)
        auto through_table = [&](const float (&acc)[KR], float2 (&v)[16]) {
            if (rm) {
                unsigned int m = rm;
#pragma unroll
                for (int i = 0; i < KR; ++i) {
                    const int r = __builtin_ctz(m);                       // KR bits are set
                    m &= m - 1;
                    part[r * kPartStride + lane] = acc[i];
                }
            }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int q = 0; q < 16; ++q) v[q] = float2{0.f, 0.f};
            if (r_out < p.BR) {
                if (p.BR <= 16) {
                    const float2 *src = reinterpret_cast<const float2 *>(part + r_out * kPartStride + grp * 16);
#pragma unroll
                    for (int q = 0; q < 8; ++q) v[q] = src[q];
                } else {
                    const float2 *src = reinterpret_cast<const float2 *>(part + r_out * kPartStride + grp * 32);
#pragma unroll
                    for (int q = 0; q < 16; ++q) v[q] = src[q];
                }
            }
            __builtin_amdgcn_wave_barrier();
        };
        // the row's sum in the fixed order of the one-step kernel (adding the zeros of the unused half changes nothing)
        auto row_sum = [&](const float2 (&v)[16]) {
            float s = 0.f;
            if (p.BR <= 16) {
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    s += v[q].x;
                    s += v[q].y;
                }
                const float s2 = s + __shfl_xor(s, 16);
                return s2 + __shfl_xor(s2, 32);
            }
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                s += v[q].x;
                s += v[q].y;
            }
            return s + __shfl_xor(s, 32);
        };
        for (int bs = 0; bs < B; bs += NS) {
            float acc[NS][KR];
            float2 v[NS][16];
#pragma unroll
            for (int s = 0; s < NS; ++s) products(bs + s < B ? bs + s : B - 1, acc[s]);      // (an odd last pass repeats a sequence)
#pragma unroll
            for (int s = 0; s < NS; ++s) through_table(acc[s], v[s]);
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                const float rs = row_sum(v[s]);
                if (bs + s < B && grp == 0 && r_out < p.BR) gl[((bs + s) * NWV + wave) * 32 + r_out] = rs;
            }
        }
        __syncthreads();

        // ---- 3. the cell on this workgroup's BR units, two sequences per thread; publish h_{t+1} under tag t + 1
        if (cell_thread) {
            unsigned int pair = 0;
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int bb = 2 * cq + k;
                if (bb < B) {
                    const float *g = gl + bb * NWV * 32 + cu;
                    float h;
                    if constexpr (CELL == 1) {
                        h = lstm_cell_apply(g[0] + b[0], g[32] + b[1], g[64] + b[2], g[96] + b[3], st[k]);
                    } else {
                        h = gru_cell_apply(g[0] + b[0], g[32] + b[1], g[64] + b[2], g[96] + b[3], g[128] + b[4], g[160] + b[5], st[k]);
                        st[k] = h;
                    }
                    const unsigned short hr = seq_round<DT>(h);
                    pair |= (unsigned int)hr << (16 * k);
                    static_cast<unsigned short *>(p.hs)[((int64_t)t * p.B + b0 + bb) * p.ldhs + ju] = hr;
                    if (p.hs32) p.hs32[((int64_t)t * p.B + b0 + bb) * p.ldhs32 + ju] = h;
                }
            }
            const unsigned long long word = (unsigned long long)pair | ((unsigned long long)(unsigned int)(t + 1) << 32);
            __hip_atomic_store(exch + ((size_t)((t + 1) & 1) * NQ + cq) * H + ju, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }

    if (gave_up) {
        if (cell_thread) {
            const unsigned long long word = (unsigned long long)kSeqPoison << 32;
            __hip_atomic_store(exch + (size_t)cq * H + ju, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(exch + ((size_t)NQ + cq) * H + ju, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (tid == 0) __hip_atomic_store(p.status, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    if (cell_thread) {
#pragma unroll
        for (int k = 0; k < 2; ++k)
            if (2 * cq + k < B) p.state[(int64_t)(b0 + 2 * cq + k) * H + ju] = st[k];
    }
}

// zeroes the exchange words' tags and the status word (a kernel, not a memset: callers may capture the launch)
__global__ void __launch_bounds__(256) rnn_seq_clear(unsigned long long *exch, int64_t words, int32_t *status) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < words) exch[i] = 0ull;
    if (i == 0) *status = 0;
}

template <int DT, int KR, int KC, int CELL, bool MULTI>
static grim_status launch_seq_inst(const SeqParams &p, dim3 grid, size_t lds, hipStream_t stream) {
    auto kern = bcr_rnn_seq<DT, KR, KC, CELL, MULTI>;
    static std::atomic<bool> attr_done{false};
    if (lds > 64 * 1024 && !attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSeqMaxLds) != hipSuccess) {
            (void)hipGetLastError();
            return GRIM_ERR_DEVICE;
        }
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(exact_waves(CELL) * 64), lds, stream, p);
    return hipGetLastError() == hipSuccess ? GRIM_OK : GRIM_ERR_DEVICE;
}

template <int DT, int CELL>
static grim_status launch_seq(const SeqParams &p, int kr, int kc, dim3 grid, size_t lds, hipStream_t stream) {
#define GRIM_SEQ(R, C)                                                                                   \
    if (kr == (R) && kc == (C))                                                                          \
        return p.SPB > 1 ? launch_seq_inst<DT, R, C, CELL, true>(p, grid, lds, stream)                   \
                         : launch_seq_inst<DT, R, C, CELL, false>(p, grid, lds, stream);
    GRIM_SEQ(4, 4) GRIM_SEQ(4, 8) GRIM_SEQ(4, 12) GRIM_SEQ(4, 16)
    GRIM_SEQ(8, 4) GRIM_SEQ(8, 8) GRIM_SEQ(8, 12) GRIM_SEQ(8, 16)
    GRIM_SEQ(16, 4) GRIM_SEQ(16, 8) GRIM_SEQ(16, 12)
#undef GRIM_SEQ
    return GRIM_ERR_UNSUPPORTED;
}

static bool seq_pair_compiled(int kr, int kc) {
    return (kr == 4 || kr == 8 || kr == 16) && (kc == 4 || kc == 8 || kc == 12 || kc == 16) && !(kr == 16 && kc == 16);
}

static size_t seq_lds_bytes(int kind, int64_t K1, int64_t K2, int BR, int batch) {
    const size_t x = ((size_t)batch * K1 * 2 + 15) & ~size_t(15), h = kind == 2 ? (((size_t)batch * K2 * 2 + 15) & ~size_t(15)) : 0;
    const size_t table = ((size_t)BR * kPartStride * 4 + 15) & ~size_t(15);
    return x + h + exact_waves(kind) * (table + (size_t)batch * 32 * 4);
}

static int compute_units() {
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

// `batch` sequences on H / BR workgroups per set: as many sets as the compute units hold (at most one per sequence),
// then several sequences per workgroup
static void seq_split(int64_t H, int BR, int batch, int cus, int *sets, int *per_wg) {
    const int64_t wgs = H / BR;
    int g = (int)std::min<int64_t>(batch, std::max<int64_t>(1, cus / wgs));
    const int spb = (batch + g - 1) / g;
    *per_wg = spb;
    *sets = (batch + spb - 1) / spb;
}

// kind 1: LSTM (K1 = I + H), kind 2: GRU (K1 = I, K2 = H).  The matrices qualify when they hold two-byte elements in
// blocks of at most 32 x 32 that all keep one compiled (rows, columns) pair, a strip has at most 64 column blocks
// (a lane keeps one block), H is a multiple of BR and one workgroup per BR hidden units fits the GPU at once; 1 .. 32
// sequences side by side whose vectors fit LDS.
bool rnn_seq_applies(int kind, int32_t BR, int32_t BC, int32_t dtype, int32_t ukr, int32_t ukc, int64_t K1, int64_t K2,
                     int64_t I, int64_t H, int32_t batch) {
    if (kind != 1 && kind != 2) return false;
    if (batch < 1 || batch > kSeqMaxBatch) return false;
    if ((dtype != GRIM_F16 && dtype != GRIM_BF16) || BR < 1 || BR > 32 || BC < 1 || BC > 32) return false;
    if (!seq_pair_compiled(ukr, ukc) || ukr > BR || ukc > BC) return false;
    if (H < 1 || I < 1 || H % BR != 0 || H > kSeqMaxH) return false;
    if (kind == 1 ? K1 != I + H : (K1 != I || K2 != H)) return false;
    if (K1 % BC != 0 || K1 / BC > 64 || (kind == 2 && (K2 % BC != 0 || K2 / BC > 64))) return false;
    const int cus = compute_units();
    if (cus < 1 || H / BR > cus) return false;
    int sets, per_wg;
    seq_split(H, BR, batch, cus, &sets, &per_wg);
    // a cell thread per hidden unit and pair of the workgroup's sequences
    if ((int64_t)BR * ((per_wg + 1) / 2) > exact_waves(kind) * 64) return false;
    return seq_lds_bytes(kind, K1, K2, BR, per_wg) <= kSeqMaxLds;
}

grim_status launch_rnn_seq(int kind, const GemvDesc &d1, const GemvDesc *d2, const int32_t *pos1, const int32_t *pos2,
                           int32_t BR, int32_t BC, int32_t dtype, int32_t ukr, int32_t ukc, int64_t K1, int64_t K2, int64_t I,
                           int64_t H, int32_t T, int32_t batch, const void *xs, int64_t ldxs, const void *h0, const float *bias,
                           const float *bias2, float *state, void *hs, int64_t ldhs, float *hs32, int64_t ldhs32,
                           void *exch, int32_t *status, uint32_t max_polls, hipStream_t stream) {
    if ((kind == 2 && (!d2 || !pos2)) || !rnn_seq_applies(kind, BR, BC, dtype, ukr, ukc, K1, K2, I, H, batch)) return GRIM_ERR_UNSUPPORTED;
    if (T < 1 || ldxs < I || ldhs < H || (hs32 && ldhs32 < H)) return GRIM_ERR_SHAPE;
    if ((int64_t)T * batch > 0x7fffffff) return GRIM_ERR_SHAPE;
    SeqParams p;
    p.d1 = d1;
    p.d2 = d2 ? *d2 : d1;
    p.pos1 = pos1;
    p.pos2 = pos2 ? pos2 : pos1;
    p.BR = BR; p.BC = BC;
    p.nbc1 = (int32_t)(K1 / BC);
    p.nbc2 = kind == 2 ? (int32_t)(K2 / BC) : p.nbc1;
    p.K1 = (int32_t)K1; p.K2 = (int32_t)K2;
    p.I = (int32_t)I; p.H = (int32_t)H; p.T = T;
    int sets = 1, per_wg = 1;
    seq_split(H, BR, batch, compute_units(), &sets, &per_wg);
    p.B = batch; p.SPB = per_wg; p.NQ = (per_wg + 1) / 2;
    // pieces a thread fetches ahead: one when a workgroup carries one sequence, up to kSeqXVec otherwise
    p.xvec16 = (I % 8 == 0 && K1 % 8 == 0 && per_wg * (I / 8) <= (per_wg > 1 ? kSeqXVec : 1) * exact_waves(kind) * 64 &&
                ldxs % 8 == 0 && reinterpret_cast<uintptr_t>(xs) % 16 == 0) ? 1 : 0;
    p.xs = xs; p.ldxs = ldxs; p.h0 = h0;
    p.bias = bias; p.bias2 = bias2;
    p.state = state;
    p.hs = hs; p.ldhs = ldhs; p.hs32 = hs32; p.ldhs32 = ldhs32;
    p.exch = static_cast<unsigned long long *>(exch);
    p.status = status;
    p.max_polls = max_polls ? max_polls : kSeqDefaultPolls;
    const int64_t words = (int64_t)sets * 2 * p.NQ * H;                // at most 2 * kSeqMaxBatch * H
    hipLaunchKernelGGL(rnn_seq_clear, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, stream, p.exch, words, status);
    if (hipGetLastError() != hipSuccess) return GRIM_ERR_DEVICE;
    const dim3 grid((unsigned)(H / BR), (unsigned)sets);
    const size_t lds = seq_lds_bytes(kind, K1, K2, BR, per_wg);
    if (kind == 1)
        return dtype == GRIM_F16 ? launch_seq<GRIM_F16, 1>(p, ukr, ukc, grid, lds, stream)
                                 : launch_seq<GRIM_BF16, 1>(p, ukr, ukc, grid, lds, stream);
    return dtype == GRIM_F16 ? launch_seq<GRIM_F16, 2>(p, ukr, ukc, grid, lds, stream)
                             : launch_seq<GRIM_BF16, 2>(p, ukr, ukc, grid, lds, stream);
}

// Exchange words for callers that must not allocate: one array per GPU, part of the loaded code object, shared by
// every such call on that GPU (calls that overlap in time on one GPU race).  Its name is a host-side stand-in; the
// device address is asked for once per device, with that device current, and only that address is handed to kernels.
static __device__ __align__(256) unsigned long long scratch[2 * kSeqMaxH];

grim_status rnn_seq_static_exchange(void **out) {
    constexpr int kMaxDevices = 64;
    static std::mutex lock;
    static void *address[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return GRIM_ERR_DEVICE;
    }
    std::lock_guard<std::mutex> hold(lock);
    if (!address[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return GRIM_ERR_DEVICE;
        }
        address[dev] = ptr;
    }
    *out = address[dev];
    return GRIM_OK;
}

}  // namespace grim

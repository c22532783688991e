// Wide-tile staged matrix-core SpMM kernel (fp16 / bf16, BR = 16 or 32) for Y = W_bcr * X with many columns
// (Section 3.1: a CONV layer at a large batch or resolution; Section 4.4: tiling, and the rows of X a block keeps
// loaded once and reused by all of its kept rows).
//
// The product streams X exactly once, so the design goal is one round of fat workgroups that keep HBM busy:
//   * a workgroup owns a tile of 96-192 columns of X and 16 row strips: eight multiplying waves, two strips
//     each, and four fetching waves -- twelve waves, three per SIMD, 168 registers each: room for 96
//     accumulators and two sets of operand fragments in a multiplying wave, for two chunks of loads in flight
//     in a fetching wave;
//   * K is cut into chunks of at most 128 rows (192 for the 96-column tiles of BR = 32).  The fetching waves move the rows of the tile and the step
//     records of the group's strips global -> registers -> LDS; a chunk's rows are asked for two chunks before they
//     are written to LDS and three before they are multiplied, so that HBM latency spans two chunk periods; LDS
//     holds two stages, one barrier per chunk.  Fetching runs under the multiplies of the chunk before;
//   * a multiplying wave walks the steps of both of its strips in a chunk as one list with a software pipeline
//     one step deep: the LDS transpose reads (the gather of the kept rows straight into MFMA operand layout)
//     and the weight read of the next step are issued before the current step is multiplied.  Lanes of rows a
//     block does not keep multiply zeros, so sums land at strip positions and the scatter needs no pass of its own.
// Record format and step layout are those of the staged kernel (bcr_matrix.hpp), cut for these shorter chunks.
// Accumulation is fp32 in a fixed order, no atomics.
#include <algorithm>

#include "spmm_common.hpp"

namespace grim {

struct WideParams {
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
};

constexpr int kWideMulWaves = 8;     // multiplying waves, two strips each
constexpr int kWideFetchWaves = 4;   // fetching waves
constexpr int kWideThreads = (kWideMulWaves + kWideFetchWaves) * 64;
constexpr int kWideFetchThreads = kWideFetchWaves * 64;
constexpr int kWideStrips = 2 * kWideMulWaves;   // strips per workgroup
// 16-byte record units per fetching thread and chunk: 8 = 32 KB per (chunk, group), the layout's limit; the
// 192-column shape, whose rows of X take more registers, has room for 4 (16 KB)
constexpr int wide_sru(int tn) { return tn == 192 ? 4 : 8; }
static_assert(wide_sru(128) * kWideFetchThreads * 16 == kWideMaxRecordBytes, "record staging registers cover the layout's limit");

// Rows of a stage are padded by 32 bytes: consecutive rows then start 32 bytes apart modulo the 256-byte bank line
// (pitches 224, 288 and 416 give eight distinct offsets), so the four rows one transpose read gathers -- 32 bytes
// of each -- spread over the banks without a swizzle, and the addresses of a row's sub-tiles differ by constants.
constexpr int kWidePad = 32;

__host__ __device__ inline int wide_stage_bytes(int chunk_rows, int tn, int amax) {
    return (chunk_rows + 1) * (tn * 2 + kWidePad) + amax * 16;
}

// third dword of a raw buffer descriptor on this GPU family (32-bit data format); only the range check matters here
constexpr unsigned int kBufferFlags = 0x00020000u;

// BR = 16: v_mfma_f32_16x16x32, product taken as (X^T tile) x (W^T fragment): a lane ends with 4 consecutive
//          columns of one output row.  BR = 32: v_mfma_f32_32x32x16, weights first: a lane holds one column, 16 rows.
template <bool BF16, int BR, int NT>
__global__ void __launch_bounds__(kWideThreads) bcr_spmm_wide(WideParams p) {
    constexpr int NSUB = BR == 16 ? 16 : 32;
    constexpr int TN = NT * NSUB;
    constexpr int PITCH = TN * 2 + kWidePad;     // LDS row pitch in bytes
    constexpr int CPR = TN / 8;                  // 16-byte units per staged row
    constexpr int NTB = NT == 12 ? 3 : NT % 4 == 0 ? 4 : 3;   // sub-tiles per pipeline item
    constexpr int NB = NT / NTB;                 // items per step
    constexpr int KS = BR == 16 ? 32 : 16;       // k slots per step
    constexpr int HDR = KS * 2 + (KS / 8) * 8;   // header bytes per step
    constexpr int SXU = (wide_max_chunk_rows(BR) * CPR + kWideFetchThreads - 1) / kWideFetchThreads;   // X units per fetching thread and chunk
    constexpr int NW = kWideMulWaves;
    constexpr int SRU = wide_sru(TN);
    static_assert(NT % NTB == 0, "sub-tiles come in whole batches");
    using Acc = typename std::conditional<BR == 16, f32x4, f32x16>::type;

    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int xbytes = (p.chunk_rows + 1) * PITCH;            // X rows + zero row
    const int stage_bytes = xbytes + p.amax * 16;

    // workgroup -> (tile, strip group).  Workgroup ids are dealt to the 8 XCDs round-robin and each XCD has its own L2:
    // all groups of a tile run on the same XCD, and so do tiles 2 k and 2 k + 1 -- a 96-column tile is one and a half
    // 128-byte lines wide, so these two share a line of every row, which the pair then takes from HBM once.
    const int id = blockIdx.x;
    const int xcd = id & 7, slot = id >> 3;
    const int tslot = slot / p.ngroups;
    const int tile = (tslot >> 1) * 16 + xcd * 2 + (tslot & 1);
    const int group = slot % p.ngroups;
    if (tile >= p.ntiles) return;
    // a ragged last tile is shifted left to end at N (N >= TN, N a multiple of 8: checked at launch); it overlaps
    // its neighbour and both write the same bits to the shared columns
    int64_t n0 = (int64_t)tile * TN;
    if (n0 + TN > p.N) n0 = p.N - TN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // The two step tables are read with wave-uniform indices only; named in the constant address space they are
    // fetched through the scalar cache into scalar registers (they are never written while a kernel runs).
    using Table = const __attribute__((address_space(4))) int32_t *;
    const Table cptr = (Table)p.cptr, bptr = (Table)p.bptr;
    const int t0 = group * kWideStrips;
    const int t1 = t0 + kWideStrips < p.nbr ? t0 + kWideStrips : p.nbr;

    if (wave >= NW) {
        // ------------------------------------------------------------------ fetching waves
        const int ft = tid - NW * 64;            // 0 .. 255
        // zero rows (gather target of padded k slots), one per stage
        static_assert(2 * (PITCH / 4) <= kWideFetchThreads, "one thread per dword of the two zero rows");
        if (ft < 2 * (PITCH / 4)) {
            const int st = ft / (PITCH / 4), w = ft % (PITCH / 4);
            *reinterpret_cast<unsigned int *>(lds + st * stage_bytes + p.chunk_rows * PITCH + w * 4) = 0u;
        }
        // The thread's i-th unit of a chunk is unit i * 256 + ft = (row of the chunk, 16-byte piece of the row).
        // All loads are buffer loads, always issued: a row past the end of K or a record unit past the end of the
        // group's records is out of the buffer's range and reads zeros without a fetch -- no conditional load
        // anywhere, so a wait for an older set of loads never has to assume that the younger set is missing.
        int xoff[SXU];
#pragma unroll
        for (int i = 0; i < SXU; ++i) {
            const int u = i * kWideFetchThreads + ft;
            const int row = u / CPR, c = u - row * CPR;
            xoff[i] = (int)(row * p.ldx * 2 + c * 16);      // below 2^31: checked at launch
        }
        // rows 0 .. K - 1 of the tile's columns: the last valid byte is the end of row K - 1's piece
        const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<unsigned short *>(p.X + n0), 0, (int)(((int64_t)(p.K - 1) * p.ldx + TN) * 2), kBufferFlags);
        u32x4 RX0[SXU], RX1[SXU], RR[SRU];
        // (past the last chunk the last one is fetched again and never stored)
        auto load_records = [&](int chunk, u32x4 (&rr)[SRU]) {
            chunk = chunk < p.nchunks ? chunk : p.nchunks - 1;
            const Table bp = bptr + (int64_t)chunk * (p.nbr + 1);
            const int b0 = __builtin_amdgcn_readfirstlane(bp[t0]), units = __builtin_amdgcn_readfirstlane(bp[t1]) - b0;
            const __amdgpu_buffer_rsrc_t rres = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<unsigned char *>(p.recs) + (int64_t)b0 * 16, 0, units * 16, kBufferFlags);
#pragma unroll
            for (int i = 0; i < SRU; ++i)
                rr[i] = __builtin_amdgcn_raw_buffer_load_b128(rres, (i * kWideFetchThreads + ft) * 16, 0, 0);
        };
        auto load_rows = [&](int chunk, u32x4 (&rx)[SXU]) {
            chunk = chunk < p.nchunks ? chunk : p.nchunks - 1;
            const int soff = __builtin_amdgcn_readfirstlane((int)((int64_t)chunk * p.chunk_rows * p.ldx * 2));
#pragma unroll
            for (int i = 0; i < SXU; ++i) rx[i] = __builtin_amdgcn_raw_buffer_load_b128(xres, xoff[i], soff, 0);
        };
        auto store_records = [&](int chunk, const u32x4 (&rr)[SRU]) {
            char *sbase = lds + (chunk & 1) * stage_bytes + xbytes;
            const Table bp = bptr + (int64_t)chunk * (p.nbr + 1);
            const int units = bp[t1] - bp[t0];
#pragma unroll
            for (int i = 0; i < SRU; ++i) {
                const int u = i * kWideFetchThreads + ft;
                if (u < units) *reinterpret_cast<u32x4 *>(sbase + u * 16) = rr[i];
            }
        };
        auto store_rows = [&](int chunk, const u32x4 (&rx)[SXU]) {
            char *sbase = lds + (chunk & 1) * stage_bytes;
            int fo = ft;
            asm volatile("" : "+v"(fo));         // the unit addresses are recomputed here, not held in registers across the loop
#pragma unroll
            for (int i = 0; i < SXU; ++i) {
                const int u = i * kWideFetchThreads + fo;
                const int row = u / CPR, c = u - row * CPR;
                if (row < p.chunk_rows) *reinterpret_cast<u32x4 *>(sbase + row * PITCH + c * 16) = rx[i];
            }
        };
        // Chunk c is multiplied from stage c % 2 while chunk c + 1 is written to the other stage (read last in chunk
        // c - 1).  Rows of X come from HBM: two register sets, a chunk's rows are asked for two chunks before they are
        // written.  Records come from L2: one set, asked for one chunk ahead, and always BEFORE the rows asked for in
        // the same period, so that the wait for them (loads return in order) leaves those younger rows in flight.
        load_rows(0, RX0);
        load_records(0, RR);
        store_rows(0, RX0);
        store_records(0, RR);
        load_records(1, RR);
        load_rows(1, RX1);
        load_rows(2, RX0);
        __syncthreads();
        for (int c = 0; c < p.nchunks; c += 2) {
            if (c + 1 < p.nchunks) { store_rows(c + 1, RX1); store_records(c + 1, RR); }
            load_records(c + 2, RR);
            load_rows(c + 3, RX1);
            __syncthreads();
            if (c + 1 >= p.nchunks) break;
            if (c + 2 < p.nchunks) { store_rows(c + 2, RX0); store_records(c + 2, RR); }
            load_records(c + 3, RR);
            load_rows(c + 4, RX0);
            __syncthreads();
        }
        return;
    }

    // ---------------------------------------------------------------------- multiplying waves
    Acc acc[2][NT];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int q = 0; q < NT; ++q)
#pragma unroll
            for (int e = 0; e < (BR == 16 ? 4 : 16); ++e) acc[s][q][e] = 0.f;

    // per-lane constants of the gather: byte column inside a sub-tile
    const int i16 = lane & 15;
    const int ncolb = ((BR == 16 ? 0 : 16 * ((lane >> 4) & 1)) + 4 * (i16 & 3)) * 2;
    // per-lane constants of the weight fragment: output row inside the strip and k group
    const int m_row = BR == 16 ? (lane & 15) : (lane & 31);
    const int kgroup = BR == 16 ? (lane >> 4) : (lane >> 5);
    const unsigned int below = (1u << m_row) - 1u, mybit = 1u << m_row;
    const int hdr_rows = (kgroup * 4 + (i16 >> 2)) * 4;        // this lane's pair of staged-row numbers
    const int hdr_desc = KS * 2 + kgroup * 8;                  // its group's (row mask, payload offset)
    // stored strips of this wave: strips are stored by decreasing work, so the wave with the k-th heaviest strip of the
    // group's first half takes the k-th lightest of the second half
    const int tA = t0 + wave, tB = t0 + 2 * NW - 1 - wave;

    struct Hdr { unsigned int rr; uint2 dsc; };
    auto load_hdr = [&](const char *h) {
        Hdr f;
        f.rr = *reinterpret_cast<const unsigned int *>(h + hdr_rows);
        f.dsc = *reinterpret_cast<const uint2 *>(h + hdr_desc);
        return f;
    };
    auto load_x = [&](const char *stage, const Hdr &f, int b, i16x8 (&x)[NTB]) {
        const int r0 = f.rr & 0xffff, r1 = f.rr >> 16;
        const char *x0 = stage + r0 * PITCH + ncolb;
        const char *x1 = stage + r1 * PITCH + ncolb;
#pragma unroll
        for (int j = 0; j < NTB; ++j) {
            const int qoff = (b * NTB + j) * NSUB * 2;            // a constant: folded into the read's offset field
            const i16x4 lo = lds_tr_read(x0 + qoff);
            const i16x4 hi = lds_tr_read(x1 + qoff);
            x[j] = i16x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        }
    };

    // (steps, region offset) of the wave's two strips in a chunk -- wave-uniform, read through the scalar cache
    struct Entry { int nA, nB, offA, offB; };
    auto entry_of = [&](int ch) {
        const Table cp = cptr + (int64_t)ch * (p.nbr + 1), bp = bptr + (int64_t)ch * (p.nbr + 1);
        const int a0 = tA < p.nbr ? tA : p.nbr, a1 = tA + 1 < p.nbr ? tA + 1 : p.nbr;
        const int b0 = tB < p.nbr ? tB : p.nbr, b1 = tB + 1 < p.nbr ? tB + 1 : p.nbr;
        const int base = bp[t0];
        Entry e;
        e.nA = cp[a1] - cp[a0];
        e.nB = cp[b1] - cp[b0];
        e.offA = (bp[a0] - base) * 16;
        e.offB = (bp[b0] - base) * 16;
        return e;
    };

    // A pipeline item is (step, batch of NTB sub-tiles).  The loads of the next item -- for a new step its weights, its
    // gathered rows and the header of the step after it -- are issued BEFORE the current item is multiplied and land in
    // a second set of registers; items are taken in pairs so that the two sets swap roles without a copy (a copy
    // would wait for the load it copies).  The scheduling barriers keep the compiler from moving the multiplies ahead
    // of the loads: the LDS round trip of one item has to run under the multiplies of the item before it.  Whether
    // a lane's row is kept is applied to its weights only when they are used.
    struct Frag { i16x8 x[NTB]; i16x8 w; unsigned int kept; };
    auto compute = [&](int ch, const Entry &en) {
        const int n = en.nA + en.nB;
        if (n <= 0) return;
        const char *stage = lds + (ch & 1) * stage_bytes;
        const char *regA = stage + xbytes + en.offA, *regB = stage + xbytes + en.offB;
        // virtual step v of the wave's list: strip A's steps, then strip B's (clamped to the last one)
        auto region_of = [&](int v) { return v < en.nA ? regA : regB; };
        auto hdr_of = [&](int v) {
            v = v < n ? v : n - 1;
            return v < en.nA ? regA + v * HDR : regB + (v - en.nA) * HDR;
        };
        // item it = v * NB + b
        auto issue = [&](int it, const Hdr &h, const Frag &prev, Frag &f) {
            const int b = it % NB;
            if (b == 0) {
                int v = it / NB;
                const bool past = v >= n;                 // a step past the list: any valid loads, zero weights
                v = past ? n - 1 : v;
                const char *region = region_of(v);
                f.kept = past ? 0u : h.dsc.x & mybit;
                const int idx = f.kept ? __builtin_popcount(h.dsc.x & below) : 0;
                f.w = *reinterpret_cast<const i16x8 *>(region + (h.dsc.y + idx) * 16);
            } else {
                f.kept = prev.kept;
                f.w = prev.w;
            }
            load_x(stage, h, b, f.x);
        };
        auto multiply = [&](Acc (&a)[NT], int b, const Frag &f) {
            const i16x8 w = f.kept ? f.w : i16x8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int j = 0; j < NTB; ++j) {
                if constexpr (BR == 16) a[b * NTB + j] = mfma16<BF16>(f.x[j], w, a[b * NTB + j]);
                else a[b * NTB + j] = mfma32<BF16>(w, f.x[j], a[b * NTB + j]);
            }
        };
        Frag fa, fb;
        Hdr hc, hn;    // headers of the step of the item in flight and of the step after it
        // One step (NB items, NB even or 1) or a pair of steps (NB = 1) per block, so that every block starts with
        // fa holding the loads of its first item, hc that item's header and hn the header of the next step.
        if constexpr (NB == 1) {
            auto pair = [&](int v, Acc (&a0)[NT], Acc (&a1)[NT]) {
                hc = load_hdr(hdr_of(v + 2));
                issue(v + 1, hn, fa, fb);
                __builtin_amdgcn_sched_barrier(0);
                multiply(a0, 0, fa);
                __builtin_amdgcn_sched_barrier(0);
                hn = load_hdr(hdr_of(v + 3));
                issue(v + 2, hc, fb, fa);
                __builtin_amdgcn_sched_barrier(0);
                if (v + 1 < n) multiply(a1, 0, fb);       // (a pair may reach one step past the list)
                __builtin_amdgcn_sched_barrier(0);
            };
            hc = load_hdr(hdr_of(0));
            hn = load_hdr(hdr_of(1));
            issue(0, hc, fb, fa);
            // Steps go in pairs on every path (a separate single-step tail that updates the accumulators on one path
            // only makes the compiler keep a second copy of them); a pair that reaches one step past the list skips
            // its second multiply.
            int v = 0;
            for (; v + 1 < en.nA; v += 2) pair(v, acc[0], acc[0]);
            if (v < en.nA) {
                pair(v, acc[0], acc[1]);
                v += 2;
            }
            for (; v < n; v += 2) pair(v, acc[1], acc[1]);
        } else {
            static_assert(NB == 1 || NB % 2 == 0, "a step's items come in pairs");
            auto step = [&](int v, Acc (&a)[NT]) {
#pragma unroll
                for (int b = 0; b < NB; b += 2) {
                    issue(v * NB + b + 1, hc, fa, fb);
                    __builtin_amdgcn_sched_barrier(0);
                    multiply(a, b, fa);
                    __builtin_amdgcn_sched_barrier(0);
                    if (b + 2 < NB) {
                        issue(v * NB + b + 2, hc, fb, fa);
                    } else {
                        issue((v + 1) * NB, hn, fb, fa);          // the next step's first item
                        hc = hn;
                        hn = load_hdr(hdr_of(v + 2));
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    multiply(a, b + 1, fb);
                    __builtin_amdgcn_sched_barrier(0);
                }
            };
            hc = load_hdr(hdr_of(0));
            hn = load_hdr(hdr_of(1));
            issue(0, hc, fb, fa);
            for (int v = 0; v < en.nA; ++v) step(v, acc[0]);
            for (int v = en.nA; v < n; ++v) step(v, acc[1]);
        }
    };

    Entry en = entry_of(0);
    __syncthreads();
    for (int c = 0; c < p.nchunks; ++c) {
        const Entry en1 = entry_of(c + 1 < p.nchunks ? c + 1 : c);
        compute(c, en);
        en = en1;
        __syncthreads();
    }

    // ---- write the strip tiles of Y (original row order); streaming stores: Y is written once and not read here ----
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const int t = s == 0 ? tA : tB;
        if (t >= p.nbr) continue;
        const int64_t row0 = (int64_t)p.strip_order[t] * BR;
#pragma unroll
        for (int q = 0; q < NT; ++q) {
            if constexpr (BR == 16) {
                // D[n][m]: lane holds m = lane % 16, n = 4 * (lane / 16) + 0..3 (16-byte aligned: checked at launch)
                const int64_t n = n0 + q * 16 + 4 * (lane >> 4);
                __builtin_nontemporal_store(acc[s][q], reinterpret_cast<f32x4 *>(p.Y + (row0 + (lane & 15)) * p.ldy + n));
            } else {
                // D[m][n]: lane holds n = lane % 32, m = 8 * (e / 4) + 4 * (lane / 32) + e % 4
                const int64_t n = n0 + q * 32 + (lane & 31);
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int m = 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                    __builtin_nontemporal_store(acc[s][q][e], &p.Y[(row0 + m) * p.ldy + n]);
                }
            }
        }
    }
}

// compiled tile widths: BR = 16: 128 and 192 columns, BR = 32: 96 columns (its accumulators leave no room for more)
static bool wide_tile_ok(int BR, int tn) { return BR == 16 ? (tn == 128 || tn == 192) : BR == 32 ? tn == 96 : false; }

static int64_t wide_lds_bytes(const grim_bcr_matrix *A, int tn) {
    return 2 * (int64_t)wide_stage_bytes(A->mmaw.chunk_rows, tn, A->mmaw.amax[2]);
}

bool wide_applies(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, const float *Y, int64_t ldy, int32_t tile_n) {
    if (!A->mmaw.present || A->dtype == GRIM_F32) return false;
    if (reinterpret_cast<uintptr_t>(X) % 16 != 0 || ldx % 8 != 0 || N % 8 != 0) return false;      // 16-byte row pieces
    if (reinterpret_cast<uintptr_t>(Y) % 16 != 0 || ldy % 4 != 0) return false;                    // 16-byte stores
    if (A->mmaw.chunk_rows > wide_max_chunk_rows(A->BR)) return false;
    if (A->K * ldx * 2 >= (int64_t(1) << 31)) return false;                                        // 32-bit buffer offsets
    for (int tn : {96, 128, 192}) {
        if (tile_n && tn != tile_n) continue;
        if (wide_tile_ok(A->BR, tn) && N >= tn && wide_lds_bytes(A, tn) <= 160 * 1024 &&
            (int64_t)A->mmaw.amax[2] <= (int64_t)wide_sru(tn) * kWideFetchThreads) return true;
    }
    return false;
}

// Cost of the wide-tile kernel on n columns in tiles of tn, in the unit the other kernels' estimates use (bytes
// through one compute unit, one after the other): a workgroup streams its tile's rows of X and the records of its
// group of strips and pays a start-up (prologue of two chunks, epilogue of the Y tile); one workgroup per compute
// unit, so the launch runs in rounds of 256.
static double wide_cost(const grim_bcr_matrix *A, int tn, int64_t n) {
    const int64_t groups = (A->nbr + kWideStrips - 1) / kWideStrips;
    const int64_t nwg = (n + tn - 1) / tn * groups;
    const double rounds = (double)((nwg + 255) / 256);
    const double rec = (double)A->mmaw.recs.size() * (double)std::min<int64_t>(kWideStrips, A->nbr) / (double)A->nbr;
    return rounds * ((double)A->K * tn * 2 + rec + 150e3);
}

// The best use of the wide-tile kernel for this product: all N columns in one launch, or the leading columns that fill
// whole rounds of workgroups (a multiple of the tile width) with the remaining columns left to the other kernels
// (`rest_cost(n)` prices them).  Returns the cost and sets *tn_out and *n_main (columns for this kernel); < 0: the
// kernel does not apply.  Products with fewer than 8 strips do not share a tile's rows of X between enough strips.
double wide_plan(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, const float *Y, int64_t ldy,
                 double (*rest_cost)(const grim_bcr_matrix *, int64_t), int *tn_out, int64_t *n_main) {
    if (!wide_applies(A, X, N, ldx, Y, ldy, 0) || A->nbr < 8) return -1.0;
    const int64_t groups = (A->nbr + kWideStrips - 1) / kWideStrips;
    double best = -1.0;
    for (int tn : {192, 128, 96}) {
        if (!wide_applies(A, X, N, ldx, Y, ldy, tn)) continue;
        const double all = wide_cost(A, tn, N);
        if (best < 0 || all < best) { best = all; *tn_out = tn; *n_main = N; }
        const int64_t per_round = 256 / groups;
        const int64_t main_cols = per_round > 0 ? N / tn / per_round * per_round * tn : 0;
        if (main_cols > 0 && main_cols < N && rest_cost) {
            const double rest = rest_cost(A, N - main_cols);
            if (rest >= 0 && wide_cost(A, tn, main_cols) + rest < best) {
                best = wide_cost(A, tn, main_cols) + rest;
                *tn_out = tn;
                *n_main = main_cols;
            }
        }
    }
    return best;
}

template <bool BF16, int BR, int NT>
static grim_status launch_wide_inst(const WideParams &p, size_t lds, int64_t nwg, hipStream_t stream) {
    auto kern = bcr_spmm_wide<BF16, BR, NT>;
    static std::atomic<bool> attr_done{false};    // raising a kernel's LDS limit is needed once per process
    if (lds > 64 * 1024 && !attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) {
            (void)hipGetLastError();
            return GRIM_ERR_DEVICE;
        }
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(kWideThreads), lds, stream, p);
    return hipGetLastError() == hipSuccess ? GRIM_OK : GRIM_ERR_DEVICE;
}

grim_status launch_spmm_wide(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, float *Y, int64_t ldy,
                             int32_t tile_n, hipStream_t stream) {
    int tn = tile_n;
    if (!tn) {
        // the widest tile that leaves at least 256 workgroups, else the narrowest
        const int64_t groups = (A->nbr + kWideStrips - 1) / kWideStrips;
        for (int t : {192, 128, 96}) {
            if (!wide_applies(A, X, N, ldx, Y, ldy, t)) continue;
            tn = t;
            if ((N + t - 1) / t * groups >= 256) break;
        }
    }
    if (!tn || !wide_applies(A, X, N, ldx, Y, ldy, tn)) return GRIM_ERR_UNSUPPORTED;
    const MmaLayout &L = A->mmaw;
    WideParams p;
    p.recs = L.d_recs; p.cptr = L.d_cptr; p.bptr = L.d_bptr;
    p.strip_order = A->dev.strip_order;
    p.X = static_cast<const unsigned short *>(X);
    p.Y = Y;
    p.N = N; p.ldx = ldx; p.ldy = ldy;
    p.K = (int32_t)A->K; p.nbr = (int32_t)A->nbr; p.nchunks = L.nchunks; p.chunk_rows = L.chunk_rows;
    p.ntiles = (int32_t)((N + tn - 1) / tn);
    p.ngroups = (int32_t)((A->nbr + kWideStrips - 1) / kWideStrips);
    p.amax = L.amax[2];
    const int64_t nwg = ((int64_t)p.ntiles + 15) / 16 * 16 * p.ngroups;      // tiles are dealt to the XCDs in pairs
    if (nwg > 0x7fffffff) return GRIM_ERR_SHAPE;
    const size_t lds = (size_t)wide_lds_bytes(A, tn);
    const bool bf = A->dtype == GRIM_BF16;
    if (A->BR == 16) {
        if (tn == 128) return bf ? launch_wide_inst<true, 16, 8>(p, lds, nwg, stream) : launch_wide_inst<false, 16, 8>(p, lds, nwg, stream);
        return bf ? launch_wide_inst<true, 16, 12>(p, lds, nwg, stream) : launch_wide_inst<false, 16, 12>(p, lds, nwg, stream);
    }
    return bf ? launch_wide_inst<true, 32, 3>(p, lds, nwg, stream) : launch_wide_inst<false, 32, 3>(p, lds, nwg, stream);
}

}  // namespace grim

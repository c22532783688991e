// The wide-tile staged kernel (see bcr_spmm_wide.hip for the design): one template for the product on a matrix X in
// memory and for the convolution whose im2col matrix is never formed (CONV: the fetching waves build the rows of
// that matrix in LDS straight from the feature maps; everything after the fetch is the same).
#pragma once
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
    // ---- convolution (CONV): X is null; column n of the product is output position n % HW of image n / HW, row
    // k = cin * KK + r * kw + q of the never-formed matrix is feature map F[img][cin] shifted by kernel tap (r, q)
    const unsigned short *F;     // batch x [Cin][H][W], images f_img_stride elements apart
    int32_t H, W, HW, kh, kw, KK;
    int32_t kk_magic;            // ceil(2^31 / KK): k / KK = umulhi(2 k, magic) (k * KK < 2^31: checked at launch)
    int32_t kw_magic;            // ceil(256 / kw): tap / kw = tap * magic >> 8 (checked for every tap at launch)
    int32_t f_img_stride;        // elements
    int32_t f_total;             // elements from F to the end of the last image (f_total * 2 < 2^31)
    int64_t n_begin;             // first column of this launch (N is its end)
    int64_t y_img_stride;        // elements between the [M][ldy] outputs of two images
    const float *bias;           // M values added to every position of a row, or null
    int32_t relu, odt;           // max(., 0) after the bias; element type of Y
};

// fp32 -> bf16, round to nearest even; NaN stays NaN
__device__ __forceinline__ unsigned short wide_f32_to_bf16(float f) {
    unsigned int u = __builtin_bit_cast(unsigned int, f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

// 16 bytes of a feature map at any 2-byte alignment
struct __attribute__((packed, aligned(2))) WideWindow {
    unsigned int d[4];
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

constexpr int wide_gcd(int a, int b) { return b == 0 ? a : wide_gcd(b, a % b); }

__host__ __device__ inline int wide_stage_bytes(int chunk_rows, int tn, int amax) {
    return (chunk_rows + 1) * (tn * 2 + kWidePad) + amax * 16;
}

// third dword of a raw buffer descriptor on this GPU family (32-bit data format); only the range check matters here
constexpr unsigned int kBufferFlags = 0x00020000u;

// BR = 16: v_mfma_f32_16x16x32, product taken as (X^T tile) x (W^T fragment): a lane ends with 4 consecutive
//          columns of one output row.  BR = 32: v_mfma_f32_32x32x16, weights first: a lane holds one column, 16 rows.
// (the body as a function of the workgroup's number, so that a kernel can run other workgroups next to these)
template <bool BF16, int BR, int NT, bool CONV>
__device__ __forceinline__ void wide_body(const WideParams &p, char *lds, int block_x) {
    constexpr int NSUB = BR == 16 ? 16 : 32;
    constexpr int TN = NT * NSUB;
    constexpr int PITCH = TN * 2 + kWidePad;     // LDS row pitch in bytes
    constexpr int CPR = TN / 8;                  // 16-byte units per staged row
    constexpr int NTB = NT == 12 ? 3 : NT % 4 == 0 ? 4 : NT;  // sub-tiles per pipeline item (NT <= 3: all of them)
    constexpr int NB = NT / NTB;                 // items per step
    constexpr int KS = BR == 16 ? 32 : 16;       // k slots per step
    constexpr int HDR = KS * 2 + (KS / 8) * 8;   // header bytes per step
    constexpr int SXU = (wide_max_chunk_rows(BR) * CPR + kWideFetchThreads - 1) / kWideFetchThreads;   // X units per fetching thread and chunk
    constexpr int NW = kWideMulWaves;
    constexpr int SRU = wide_sru(TN);
    static_assert(NT % NTB == 0, "sub-tiles come in whole batches");
    using Acc = typename std::conditional<BR == 16, f32x4, f32x16>::type;

    const int xbytes = (p.chunk_rows + 1) * PITCH;            // X rows + zero row
    const int stage_bytes = xbytes + p.amax * 16;

    // workgroup -> (tile, strip group).  Workgroup ids are dealt to the 8 XCDs round-robin and each XCD has its own L2:
    // all groups of a tile run on the same XCD, and so do tiles 2 k and 2 k + 1 -- a 96-column tile is one and a half
    // 128-byte lines wide, so these two share a line of every row, which the pair then takes from HBM once.
    const int id = block_x;
    const int xcd = id & 7, slot = id >> 3;
    const int tslot = slot / p.ngroups;
    const int tile = (tslot >> 1) * 16 + xcd * 2 + (tslot & 1);
    const int group = slot % p.ngroups;
    if (tile >= p.ntiles) return;
    // a ragged last tile is shifted left to end at N (N >= TN, N a multiple of 8: checked at launch); it overlaps
    // its neighbour and both write the same bits to the shared columns
    int64_t n0 = (CONV ? p.n_begin : 0) + (int64_t)tile * TN;
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
        // The loads of the rows are buffer loads, always issued: a row past the end of K is out of the buffer's range
        // and reads zeros without a fetch -- no conditional load among them, so a wait for an older set of rows never
        // has to assume that the younger set is missing.
        // SpMM: byte offset of the unit inside the tile's columns of X.  CONV: element of F at which the unit's 8
        // positions start (image and position of the piece), to which a row of the matrix adds its channel and tap.
        // (CONV: a thread's units i, i + XP, i + 2 XP, ... are the same piece of different rows, so XP offsets do)
        constexpr int XSTEP = kWideFetchThreads % CPR;
        constexpr int XP = !CONV ? SXU : XSTEP == 0 ? 1 : (CPR / wide_gcd(CPR, XSTEP) < SXU ? CPR / wide_gcd(CPR, XSTEP) : SXU);
        int xoff[XP];
#pragma unroll
        for (int i = 0; i < XP; ++i) {
            const int u = i * kWideFetchThreads + ft;
            const int row = u / CPR, c = u - row * CPR;
            if constexpr (CONV) {
                const int64_t n = n0 + c * 8;
                const int img = (int)(n / p.HW);
                xoff[i] = img * p.f_img_stride + (int)(n - (int64_t)img * p.HW);
            } else {
                xoff[i] = (int)(row * p.ldx * 2 + c * 16);      // below 2^31: checked at launch
            }
        }
        // CONV: per (kernel tap, piece of the tile) the 16-byte mask of the positions whose shifted pixel lies inside
        // the image (a piece never straddles two images: HW is a multiple of 8); entry KK is all zero (rows past K).
        // It sits behind the two stages.
        u32x4 *vtab = reinterpret_cast<u32x4 *>(lds + 2 * stage_bytes);
        const int centre = CONV ? (p.kh >> 1) * p.W + (p.kw >> 1) : 0;
        if constexpr (CONV) {
            for (int e = ft; e < (p.KK + 1) * CPR; e += kWideFetchThreads) {
                const int tap = e / CPR, c = e - tap * CPR;
                const int r = tap / p.kw, q = tap - r * p.kw;
                const int dr = r - (p.kh >> 1), dq = q - (p.kw >> 1);
                const int64_t n = n0 + c * 8;
                const int pos = (int)(n % p.HW);
                int h = pos / p.W, w = pos - h * p.W;
                unsigned int m[4] = {0u, 0u, 0u, 0u};
                if (tap < p.KK) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const bool ok = h + dr >= 0 && h + dr < p.H && w + dq >= 0 && w + dq < p.W;
                        m[j >> 1] |= ok ? (j & 1 ? 0xffff0000u : 0x0000ffffu) : 0u;
                        if (++w == p.W) { w = 0; ++h; }
                    }
                }
                vtab[e] = u32x4{m[0], m[1], m[2], m[3]};
            }
        }
        // (channel-and-tap offset, tap) of row k of the never-formed matrix; rows past K: tap KK (masked to zero)
        auto conv_row = [&](int k, int &tap) {
            const bool past = k >= p.K;
            const unsigned int kk = past ? 0u : (unsigned int)k;
            const unsigned int cin = __umulhi(kk << 1, (unsigned int)p.kk_magic);
            const int t_ = (int)(kk - cin * (unsigned int)p.KK);
            const int r = (t_ * p.kw_magic) >> 8;
            tap = past ? p.KK : t_;
            return (int)cin * p.HW + r * p.W + (t_ - r * p.kw) - centre;
        };
        // That split is made once per row and chunk, not once per 16-byte unit: a ring of four per-chunk tables in LDS
        // (behind the mask table) holds it for the chunks whose rows are being asked for or written; one thread per row
        // fills the table of chunk c + 4 during the period of chunk c, a barrier before anyone reads it.
        constexpr int RTP = wide_max_chunk_rows(BR);
        int2 *rowtab = reinterpret_cast<int2 *>(lds + 2 * stage_bytes + (CONV ? (p.KK + 1) * CPR * 16 : 0));
        auto fill_rows = [&](int chunk) {
            if (ft < RTP) {
                int tap;
                const int eb = conv_row(chunk * p.chunk_rows + ft, tap);
                rowtab[(chunk & 3) * RTP + ft] = int2{eb, tap};
            }
        };
        if constexpr (CONV) {
            for (int ch = 0; ch < 4; ++ch) fill_rows(ch);
            __syncthreads();                     // both tables are complete before the first chunk is asked for
        }
        // rows 0 .. K - 1 of the tile's columns: the last valid byte is the end of row K - 1's piece
        const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<unsigned short *>(CONV ? p.F : p.X + n0), 0, CONV ? 16 : (int)(((int64_t)(p.K - 1) * p.ldx + TN) * 2), kBufferFlags);
        u32x4 RX0[SXU], RX1[SXU];
        // (past the last chunk the last one is fetched again and never stored)
        // where the records of the group's strips in a chunk start and how many 16-byte units they are: two table
        // reads through the scalar cache, asked for at the top of a chunk period and used at its end, so that their
        // latency runs under the period's stores
        struct RecRange { int b0, units; };
        auto rec_range = [&](int chunk) {
            chunk = chunk < p.nchunks ? chunk : p.nchunks - 1;
            const Table bp = bptr + (int64_t)chunk * (p.nbr + 1);
            RecRange r;
            r.b0 = __builtin_amdgcn_readfirstlane(bp[t0]);
            r.units = __builtin_amdgcn_readfirstlane(bp[t1]) - r.b0;
            return r;
        };
        // A chunk's records go from global memory straight into the stage's record area (no registers, no LDS store
        // instructions): a wave's load puts lane l's 16 bytes at the wave's base (in M0) + 16 l; lanes past the range's
        // end are masked off and write nothing.  The stage must be free when the load is ISSUED (see the loop below).
        // Written as assembly so that the compiler's own wait insertion does not see these loads: it would otherwise
        // drain every load of the wave before the next LDS store and before every barrier, which ends the rows'
        // two-chunk prefetch.  The waits it computes for the rows stay valid -- loads it does not know of only make a
        // wait for an older load stricter -- and the wait for the records themselves is explicit (landed_but_rows).
        const int fwave = __builtin_amdgcn_readfirstlane(ft >> 6);
        auto direct_records = [&](int chunk, const RecRange &r) {
            const int sbase = (int)(uintptr_t)(__attribute__((address_space(3))) char *)lds + (chunk & 1) * stage_bytes + xbytes;
            const unsigned char *src = p.recs + (int64_t)r.b0 * 16;
#pragma unroll
            for (int i = 0; i < SRU; ++i) {
                if (i * kWideFetchThreads < r.units) {
                    const int u = i * kWideFetchThreads + ft;
                    if (u < r.units)
                        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                                     :: "s"(sbase + (i * kWideFetchThreads + fwave * 64) * 16), "v"(src + (int64_t)u * 16)
                                     : "memory", "m0");
                }
            }
        };
        // every load of this wave has arrived (the direct ones: is in LDS) except the youngest SXU: loads return in
        // order, and a chunk's rows are at least SXU load instructions, always issued
        auto landed_but_rows = [&]() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(SXU) : "memory"); };
        auto load_rows = [&](int chunk, u32x4 (&rx)[SXU]) {
            const int chunk_u = chunk;           // (CONV: rows past the last chunk are past K: any address, never stored)
            chunk = chunk < p.nchunks ? chunk : p.nchunks - 1;
            if constexpr (CONV) {
                // the unit's 8 pixels: one 16-byte load at a 2-byte alignment, always issued, at an address clamped
                // into the batch (a window that starts before it or ends behind it is shifted into place when stored)
                // (the rows' table entries are read together, so that their LDS round trips overlap)
                int eb[SXU];
#pragma unroll
                for (int i = 0; i < SXU; ++i) eb[i] = rowtab[(chunk_u & 3) * RTP + (i * kWideFetchThreads + ft) / CPR].x;
#pragma unroll
                for (int i = 0; i < SXU; ++i) {
                    int e = xoff[i % XP] + eb[i];
                    e = e < 0 ? 0 : e > p.f_total - 8 ? p.f_total - 8 : e;
                    WideWindow wv;
                    __builtin_memcpy(&wv, reinterpret_cast<const char *>(p.F) + (unsigned int)(e * 2), 16);
                    rx[i] = u32x4{wv.d[0], wv.d[1], wv.d[2], wv.d[3]};
                }
            } else {
                const int soff = __builtin_amdgcn_readfirstlane((int)((int64_t)chunk * p.chunk_rows * p.ldx * 2));
#pragma unroll
                for (int i = 0; i < SXU; ++i) rx[i] = __builtin_amdgcn_raw_buffer_load_b128(xres, xoff[i], soff, 0);
            }
        };
        // SpMM: where in a stage the thread's units go, held in registers (a store is then one instruction); a unit of
        // a row past the chunk's last goes into the 32 padding bytes of row 0, which nobody reads -- no branch
        int saddr[CONV ? 1 : SXU];
        if constexpr (!CONV) {
#pragma unroll
            for (int i = 0; i < SXU; ++i) {
                const int u = i * kWideFetchThreads + ft;
                const int row = u / CPR, c = u - row * CPR;
                saddr[i] = row < p.chunk_rows ? row * PITCH + c * 16 : TN * 2 + (u & 1) * 16;
            }
        }
        auto store_rows = [&](int chunk, const u32x4 (&rx)[SXU]) {
            char *sbase = lds + (chunk & 1) * stage_bytes;
            int fo = ft;
            if constexpr (CONV) asm volatile("" : "+v"(fo));   // the unit addresses are recomputed here, not held in registers across the loop
            if constexpr (CONV) {
                // three units at a time: their table entries, then their masks, are read together (two dependent LDS
                // round trips per group instead of per unit)
                constexpr int G = 3;
#pragma unroll
                for (int g = 0; g < SXU; g += G) {
                    int2 ri[G];
                    u32x4 vm[G];
#pragma unroll
                    for (int j = 0; j < G; ++j) {
                        const int i = g + j < SXU ? g + j : SXU - 1;
                        ri[j] = rowtab[(chunk & 3) * RTP + (i * kWideFetchThreads + fo) / CPR];
                    }
#pragma unroll
                    for (int j = 0; j < G; ++j) {
                        const int i = g + j < SXU ? g + j : SXU - 1;
                        const int u = i * kWideFetchThreads + fo;
                        vm[j] = vtab[ri[j].y * CPR + (u - u / CPR * CPR)];
                    }
#pragma unroll
                    for (int j = 0; j < G; ++j) {
                        if (g + j < SXU) {
                            const int i = g + j;
                            const int u = i * kWideFetchThreads + fo;
                            const int row = u / CPR, c = u - row * CPR;
                            u32x4 v = rx[i];
                            const int e = xoff[i % XP] + ri[j].x;
                            const int ec = e < 0 ? 0 : e > p.f_total - 8 ? p.f_total - 8 : e;
                            const int d = e - ec;    // the pixels wanted start d elements behind (before: d < 0) the ones loaded
                            if (__builtin_amdgcn_ballot_w64(d != 0) != 0 && d != 0) {      // (rare: the first and last pixels of the batch)
                                unsigned __int128 x = (unsigned __int128)v[0] | (unsigned __int128)v[1] << 32 |
                                                      (unsigned __int128)v[2] << 64 | (unsigned __int128)v[3] << 96;
                                x = d >= 8 || d <= -8 ? (unsigned __int128)0 : d > 0 ? x >> (16 * d) : x << (16 * -d);
                                v = u32x4{(unsigned int)x, (unsigned int)(x >> 32), (unsigned int)(x >> 64), (unsigned int)(x >> 96)};
                            }
                            v = u32x4{v[0] & vm[j][0], v[1] & vm[j][1], v[2] & vm[j][2], v[3] & vm[j][3]};
                            if (row < p.chunk_rows) *reinterpret_cast<u32x4 *>(sbase + row * PITCH + c * 16) = v;
                        }
                    }
                }
            } else {
#pragma unroll
                for (int i = 0; i < SXU; ++i) *reinterpret_cast<u32x4 *>(sbase + saddr[i]) = rx[i];
            }
        };
        // Chunk c is multiplied from stage c % 2 while chunk c + 1 is written to the other stage (read last in chunk
        // c - 1, so free from the barrier that ends period c - 1).  Rows of X come from HBM: two register sets, a chunk's
        // rows are asked for two chunks before they are written.  Records come from L2 and go straight into the stage:
        // asked for at the top of the period that fills the stage, before the rows are written, and waited for (with
        // everything older, i.e. the rows asked for in the period before) ahead of the period's new row requests,
        // which therefore stay in flight across the barrier.
        RecRange rcur = rec_range(0), rnxt = rec_range(1);     // rcur: the range of the next chunk to be filled
        load_rows(0, RX0);
        direct_records(0, rcur);
        load_rows(1, RX1);
        store_rows(0, RX0);
        rcur = rnxt;
        load_rows(2, RX0);
        landed_but_rows();
        __syncthreads();
        for (int c = 0; c < p.nchunks; c += 2) {
            rnxt = rec_range(c + 2);
            if constexpr (CONV) fill_rows(c + 4);
            if (c + 1 < p.nchunks) { direct_records(c + 1, rcur); store_rows(c + 1, RX1); }
            rcur = rnxt;
            load_rows(c + 3, RX1);
            landed_but_rows();
            __syncthreads();
            // (no way out of the loop here: with one, the waits the compiler computes for the first half assume that the
            // second half's loads may not have been issued, and drain the rows asked for one period earlier; an odd
            // number of chunks ends with one idle period, for which the multiplying waves have a barrier of their own)
            rnxt = rec_range(c + 3);
            if constexpr (CONV) fill_rows(c + 5);
            if (c + 2 < p.nchunks) { direct_records(c + 2, rcur); store_rows(c + 2, RX0); }
            rcur = rnxt;
            load_rows(c + 4, RX0);
            landed_but_rows();
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

    if constexpr (CONV) __syncthreads();         // (the fetching waves' table of validity masks)
    Entry en = entry_of(0);
    __syncthreads();
    for (int c = 0; c < p.nchunks; ++c) {
        const Entry en1 = entry_of(c + 1 < p.nchunks ? c + 1 : c);
        compute(c, en);
        en = en1;
        __syncthreads();
    }
    if (p.nchunks & 1) __syncthreads();          // (the fetching waves' periods come in pairs)

    // ---- write the strip tiles of Y (original row order); streaming stores: Y is written once and not read here ----
    // CONV: the layer's epilogue (bias, rectifier, rounding to the next layer's element type); column n is position
    // n % HW of image n / HW, whose [M][ldy] output starts y_img_stride elements after the previous image's
    auto put = [&](int64_t at, float v) {
        if (!CONV || p.odt == GRIM_F32) {
            __builtin_nontemporal_store(v, &p.Y[at]);
        } else if (p.odt == GRIM_F16) {
            reinterpret_cast<_Float16 *>(p.Y)[at] = (_Float16)v;
        } else {
            reinterpret_cast<unsigned short *>(p.Y)[at] = wide_f32_to_bf16(v);
        }
    };
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
                const int64_t row = row0 + (lane & 15);
                if constexpr (CONV) {
                    const int64_t img = n / p.HW;
                    const int64_t at = img * p.y_img_stride + row * p.ldy + (n - img * p.HW);
                    f32x4 v = acc[s][q];
                    const float b = p.bias ? p.bias[row] : 0.f;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        v[e] += b;
                        if (p.relu) v[e] = v[e] > 0.f ? v[e] : 0.f;      // NaN stays NaN
                    }
                    if (p.odt == GRIM_F32) {
                        __builtin_nontemporal_store(v, reinterpret_cast<f32x4 *>(p.Y + at));
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) put(at + e, v[e]);
                    }
                } else {
                    __builtin_nontemporal_store(acc[s][q], reinterpret_cast<f32x4 *>(p.Y + row * p.ldy + n));
                }
            } else {
                // D[m][n]: lane holds n = lane % 32, m = 8 * (e / 4) + 4 * (lane / 32) + e % 4
                const int64_t n = n0 + q * 32 + (lane & 31);
                int64_t col = n;
                if constexpr (CONV) {
                    const int64_t img = n / p.HW;
                    col = img * p.y_img_stride + (n - img * p.HW);
                }
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int m = 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                    float v = acc[s][q][e];
                    if constexpr (CONV) {
                        v += p.bias ? p.bias[row0 + m] : 0.f;
                        if (p.relu) v = v > 0.f ? v : 0.f;
                    }
                    put((row0 + m) * p.ldy + col, v);
                }
            }
        }
    }
}

template <bool BF16, int BR, int NT, bool CONV = false>
__global__ void __launch_bounds__(kWideThreads) bcr_spmm_wide(WideParams p) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    wide_body<BF16, BR, NT, CONV>(p, lds, blockIdx.x);
}

}  // namespace grim

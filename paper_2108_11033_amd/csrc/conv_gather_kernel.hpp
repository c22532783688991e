// Kernel of bcr_conv.hip as a header: the wide-tile convolution's launcher builds a kernel that runs both.
#pragma once
#include "spmm_common.hpp"

namespace grim {

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
    // a convolution plan: per k slot of `rows` the tap and the window start for output position 0, already split
    // (tap << 27 | start + 2^25; tap = KK for padding slots); null: the kernel splits the row numbers itself
    const uint32_t *plan;
    int32_t batch, tiles_per_img;        // images; ntiles = batch * tiles_per_img
    int64_t f_img_stride, y_img_stride;  // elements between images of F and of Y
    // stride 1: the 64 positions of a tile are output positions.  stride 2: they are positions of the INPUT grid, of
    // which only those with even row and column are stored (output (h / 2, w / 2)); hmul = 2: the tiles walk the even
    // rows only (needs W % 8 == 0, so that a lane's 8 positions never straddle two rows), hmul = 1: all rows
    int32_t stride, hmul, Wo;
    int32_t Nv;                  // positions the tiles of one image walk: (rows walked) * W (or the end of a range)
    int32_t img0, pos_begin;     // first image of the launch; first position the tiles walk (a range of one image)
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
// MODE: 0 = row numbers split in the kernel, stride 1; 1 = a plan's words, stride 1; 2 = a plan's words, stride 2.
// Compile-time, so that the plain form carries none of the others' state in registers.
// The body as a function of the workgroup's number, so that another kernel can run such workgroups behind its own (the
// wide-tile convolution does, for the positions it leaves over).  All (LONGW ? LONGW : 4) waves call it together; `lds`:
// 8 KB per wave plus the validity table.
template <bool BF16, bool SOLO, int LONGW, int MODE>   // LONGW: 0, or the waves that split a long strip's steps (8 or 12)
__device__ __forceinline__ void conv_gather_body(const ConvParams &p, char *lds, int block_x) {
    constexpr bool EIGHT = LONGW > 0;
    constexpr bool PLAN = MODE != 0, S2 = MODE == 2;
    const int hmul = S2 ? p.hmul : 1;
    constexpr int NT = 4, TN = 64, PITCH = 128, CPR = 8;
    constexpr int SB = 3;                        // steps a wave has in flight
    constexpr int NWV = EIGHT ? LONGW : 4;       // waves of the workgroup
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int tile, unit;
    if (!xcd_map_at(p.map, block_x, p.ntiles, &tile, &unit)) return;
    // (a division by a run-time value is done on the vector ALU even for uniform operands; without the
    // readfirstlane everything derived from the image and tile numbers would live in vector registers)
    const int img_l = __builtin_amdgcn_readfirstlane(tile / p.tiles_per_img);
    tile = __builtin_amdgcn_readfirstlane(tile - img_l * p.tiles_per_img);
    const int img = img_l + p.img0;
    const unsigned short *Fimg = p.F + (int64_t)img * p.f_img_stride;
    const int t_raw = SOLO ? unit * 4 + wave : unit;
    const bool active = t_raw < p.nbr;           // SOLO: the last workgroup of a tile may have idle waves
    const int t = active ? t_raw : p.nbr - 1;
    int n0 = p.pos_begin + tile * TN;
    if (n0 + TN > p.Nv) n0 = p.Nv - TN;          // ragged last tile: overlap the neighbour
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
    const uint32_t *slots = PLAN ? p.plan : p.rows;
    unsigned int npk[SB];
    uint2 ndsc[SB];
#pragma unroll
    for (int u = 0; u < SB; ++u) {
        int st = s_beg + u;
        st = st < s_end ? st : s_end - 1;
        st = st < 0 ? 0 : st;                    // (a wave without steps: any valid step, never used)
        npk[u] = slots[(int64_t)st * 32 + (lane & 7) * 4 + ((lane >> 3) & 3)];
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
                int h = h0 * hmul, w = w0 + j;
                while (w >= p.W) { w -= p.W; h += hmul; }  // once at most for W >= 8 (positions past the last, of a small map: h >= H, never stored)
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
    const char *Fb = reinterpret_cast<const char *>(Fimg);
    const int HW = p.N, wstep = p.W - p.kw, emax = p.total - 8;
    const int centre = ph * p.W + pw;            // offset of the centre tap: window starts are relative to it
    // element (inside a channel) of the first of the 8 positions of piece cc: the position itself, or with every
    // second row skipped (2 * row * W + column)
    auto pos_off = [&](int cc) {
        const int nb = n0 + cc * 8;
        return hmul == 1 ? nb : nb + (nb / p.W) * p.W;
    };
    // Stride 1: the tile's first position goes into the (uniform) window start of a k slot and a lane adds only its
    // piece's 8 c -- this split, not the sum formed per lane, is what keeps the fetch loop within its registers.
    const int tile_pos = S2 ? pos_off(0) : n0;
    const int cofs = (S2 ? pos_off(c) - tile_pos : c * 8) - (1 << 25);     // this lane's piece, and the bias of the packed form
    const int off7 = S2 ? pos_off(7) - tile_pos : 56;                       // piece 7 relative to tile_pos
    // Windows that start at an odd element are fetched one element early and shifted (see below), which takes the
    // next piece to continue this one in memory: true unless rows are skipped
    const bool use_shift = hmul == 1;
    // can a window of this tile start before the feature map or end behind it?  (only in the first / last channel)
    const bool tile_edge = pos_off(0) < centre || pos_off(7) + 8 + centre > HW;
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
                pk[u] = slots[(int64_t)st * 32 + (lane & 7) * 4 + ((lane >> 3) & 3)];
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
                bool is_pad;
                int eb;                          // window start for the tile's first position (stride 2: for position 0)
                if constexpr (PLAN) {            // already split when the plan was made
                    is_pad = (int)(pk[u] >> 27) == p.KK;
                    eb = (int)(pk[u] & 0x7ffffffu) - (1 << 25) + tile_pos;
                    pk[u] = (pk[u] & 0xf8000000u) | (unsigned int)(eb + (1 << 25));
                } else {
                    is_pad = pk[u] == 0xffffffffu;
                    const unsigned int kk = is_pad ? 0u : pk[u];
                    // (24-bit multiplies: Cin, H * W, W and the tap numbers are all below 2^24)
                    const unsigned int cin = __umulhi(kk << 1, (unsigned int)p.kk_magic);
                    const int tap = (int)(kk - __umul24(cin, (unsigned int)p.KK));
                    const unsigned int r = __umul24((unsigned int)tap, (unsigned int)p.kw_magic) >> 8;   // tap / kw
                    // r * W + (tap - r * kw), less the centre tap's offset
                    eb = (int)__umul24(cin, (unsigned int)HW) + __mul24((int)r, wstep) + tap - centre + tile_pos;   // (W < kw: wstep < 0)
                    pk[u] = (unsigned int)(is_pad ? p.KK : tap) << 27 | (unsigned int)(eb + (1 << 25));
                }
                // A 16-byte load at an odd element (2 bytes off a dword) costs about three aligned ones in the
                // vector L1, a load that is only dword-aligned next to nothing.  A window that starts at an odd
                // element is therefore fetched one element early; when the step is written the lane shifts it
                // by 16 bits and takes its last element from the next lane's first dword.  The last lane of a
                // row piece has no such neighbour: lanes 0..31 fetch the boundary element of their k slot with
                // one extra 2-byte load per step, handed over by a lane permute.
                const int e7 = eb + off7;
                bool need = use_shift && lane < 32 && !is_pad && (e7 & 1);
                if constexpr (SAFE) need = need && e7 + 7 >= 0 && e7 + 7 < p.total;
                ext[u] = need ? (unsigned int)Fimg[e7 + 7] : 0u;
            }
            bool edge_any = false;
#pragma unroll
            for (int u = 0; u < SB; ++u) {
                vsel[u] = 0u;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    unsigned int sel;
                    const int e0 = piece(u, i, sel);
                    const int odd = use_shift ? e0 & 1 : 0;
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
                                    const int e = e0 - (use_shift ? e0 & 1 : 0) + j;
                                    const unsigned int v = e >= 0 && e < p.total ? Fimg[e] : 0u;
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
    char *Yimg = static_cast<char *>(p.Y) + (int64_t)img * p.y_img_stride * (p.odt == GRIM_F32 ? 4 : 2);
    auto store_one = [&](int64_t at, float v) {
        if (p.odt == GRIM_F32) {
            reinterpret_cast<float *>(Yimg)[at] = v;
        } else if (p.odt == GRIM_F16) {
            reinterpret_cast<_Float16 *>(Yimg)[at] = (_Float16)v;
        } else {
            reinterpret_cast<unsigned short *>(Yimg)[at] = conv_f32_to_bf16(v);
        }
    };
    auto finish = [&](int64_t row, int64_t n, f32x4 sum) {
        const float b = p.bias ? p.bias[row] : 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            sum[e] += b;
            if (p.relu) sum[e] = sum[e] > 0.f ? sum[e] : 0.f;     // NaN stays NaN
        }
        const int left = (int)(p.Nv - n);            // below 4 only in the one tile of a map of fewer than 64 positions
        if constexpr (S2) {
            // positions of the input grid: the ones with even row and column are outputs
            int hv = (int)(n / p.W), w = (int)(n - (int64_t)hv * p.W);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int h = hv * hmul;
                if (e < left && !(h & 1) && !(w & 1)) store_one(row * p.ldy + (int64_t)(h >> 1) * p.Wo + (w >> 1), sum[e]);
                if (++w == p.W) { w = 0; ++hv; }
            }
            return;
        }
        const bool vec = p.yvec == 4 && (n & 3) == 0;
        if (p.odt == GRIM_F32) {
            float *dst = reinterpret_cast<float *>(Yimg) + row * p.ldy + n;
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
            unsigned short *dst = reinterpret_cast<unsigned short *>(Yimg) + row * p.ldy + n;
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

template <bool BF16, bool SOLO, int LONGW, int MODE>
__global__ void __launch_bounds__(LONGW ? LONGW * 64 : 256, LONGW ? 1024 / (LONGW * 64) : 4) bcr_conv_gather(ConvParams p) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    conv_gather_body<BF16, SOLO, LONGW, MODE>(p, lds, blockIdx.x);
}

// which form of the kernel a launch takes, its workgroups and workgroup memory
struct ConvForm {
    bool solo;
    int longw, mode;
    int64_t nwg;
    size_t lds;
};
grim_status conv_gather_setup(const grim_bcr_matrix *A, const void *F, int32_t Cin, int32_t H, int32_t W, int32_t kh, int32_t kw,
                              const float *bias, int32_t relu, void *Y, int32_t odt, int64_t ldy, int32_t batch, int32_t stride,
                              int64_t f_img_stride, int64_t y_img_stride, const uint32_t *plan, int32_t img0, int64_t pos_begin,
                              int64_t pos_end, ConvParams *out, ConvForm *form);

}  // namespace grim

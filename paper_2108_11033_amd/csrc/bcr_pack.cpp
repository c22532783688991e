// Host side of the library: validation, compaction of the dense matrix into the
// canonical block-compact arrays, the derived device layouts, upload, and the
// extern "C" entry points.
#include <algorithm>
#include <cstring>
#include <map>
#include <memory>
#include <new>
#include <numeric>

#include "bcr_matrix.hpp"

using namespace grim;

namespace {

struct Slab {
    // one device allocation holding every array of a matrix, each 256-byte aligned
    size_t total = 0;
    size_t add(size_t bytes) {
        size_t off = total;
        total += (bytes + 255) & ~size_t(255);
        return off;
    }
};

grim_status validate_sets(int64_t nb, int32_t B, const int32_t *ptr, const uint16_t *idx) {
    if (ptr[0] != 0) return GRIM_ERR_INDEX;
    for (int64_t b = 0; b < nb; ++b) {
        int64_t lo = ptr[b], hi = ptr[b + 1];
        if (hi < lo || hi - lo > B) return GRIM_ERR_INDEX;
        if (hi > lo && idx == nullptr) return GRIM_ERR_NULL;
        for (int64_t t = lo; t < hi; ++t) {
            if (idx[t] >= B) return GRIM_ERR_INDEX;
            if (t > lo && idx[t] <= idx[t - 1]) return GRIM_ERR_INDEX;
        }
    }
    return GRIM_OK;
}

// ---- derived layout: matrix-core SpMM ---------------------------------------------------

bool build_mma_layout_for(grim_bcr_matrix *A, MmaLayout &L, int32_t chunk_blocks, int32_t max_chunk_rows, int gsel,
                          int64_t max_group_bytes) {
    L.chunk_blocks = chunk_blocks;
    L.chunk_rows = L.chunk_blocks * A->BC;
    L.nchunks = (int32_t)((A->nbc + L.chunk_blocks - 1) / L.chunk_blocks);
    L.ks = A->BR == 16 ? 32 : 16;
    const int32_t ng = L.ks / 8;                       // groups of 8 k slots per step
    const int32_t hdr = L.ks * 2 + ng * 8;             // header bytes per step (a multiple of 16)
    L.cptr.assign((size_t)L.nchunks * (A->nbr + 1), 0);
    L.bptr.assign((size_t)L.nchunks * (A->nbr + 1), 0);
    L.recs.clear();
    struct Group { int64_t t; int32_t j0; };           // stored block (-1: empty), first kept-column position
    std::vector<Group> groups;
    int64_t step = 0;
    const uint16_t *w = reinterpret_cast<const uint16_t *>(A->weights.data());
    const uint16_t zero_row = (uint16_t)L.chunk_rows;
    for (int32_t ch = 0; ch < L.nchunks; ++ch) {
        const int64_t c0 = (int64_t)ch * L.chunk_blocks, c1 = std::min<int64_t>(A->nbc, c0 + L.chunk_blocks);
        for (int64_t st = 0; st < A->nbr; ++st) {
            L.cptr[(size_t)ch * (A->nbr + 1) + st] = (int32_t)step;
            L.bptr[(size_t)ch * (A->nbr + 1) + st] = (int32_t)(L.recs.size() / 16);
            groups.clear();
            for (int64_t c = c0; c < c1; ++c) {
                const int64_t t = st * A->nbc + c;
                const int32_t kr = A->row_ptr[t + 1] - A->row_ptr[t], kc = A->col_ptr[t + 1] - A->col_ptr[t];
                if (kr == 0 || kc == 0) continue;       // nothing to multiply
                for (int32_t j0 = 0; j0 < kc; j0 += 8) groups.push_back({t, j0});
            }
            while (groups.size() % ng) groups.push_back({-1, 0});
            const size_t nst = groups.size() / ng;
            const size_t region0 = L.recs.size();
            L.recs.resize(region0 + nst * hdr, 0);
            uint32_t pay16 = (uint32_t)(nst * hdr / 16);    // next free payload unit, from the region start
            for (size_t q = 0; q < groups.size(); ++q) {
                const Group &gp = groups[q];
                const size_t sidx = q / ng, g = q % ng;
                unsigned char *h = L.recs.data() + region0 + sidx * hdr;
                uint16_t rows[8];
                uint32_t rowmask = 0, off = 0;
                int32_t kr = 0, kc = 0;
                int64_t c = 0;
                if (gp.t >= 0) {
                    kr = A->row_ptr[gp.t + 1] - A->row_ptr[gp.t];
                    kc = A->col_ptr[gp.t + 1] - A->col_ptr[gp.t];
                    c = gp.t % A->nbc;
                    for (int32_t qq = A->row_ptr[gp.t]; qq < A->row_ptr[gp.t + 1]; ++qq) rowmask |= 1u << A->row_idx[qq];
                }
                for (int32_t e = 0; e < 8; ++e)
                    rows[e] = (gp.t >= 0 && gp.j0 + e < kc)
                                  ? (uint16_t)((c - c0) * A->BC + A->col_idx[A->col_ptr[gp.t] + gp.j0 + e])
                                  : zero_row;
                // slot rows: quad qd of the group pairs slot qd with slot qd + 4
                uint16_t *hs = reinterpret_cast<uint16_t *>(h) + g * 8;
                for (int32_t qd = 0; qd < 4; ++qd) {
                    hs[2 * qd] = rows[qd];
                    hs[2 * qd + 1] = rows[qd + 4];
                }
                if (gp.t >= 0) {
                    off = pay16;
                    const size_t p0 = L.recs.size();
                    L.recs.resize(p0 + (size_t)kr * 16, 0);
                    h = L.recs.data() + region0 + sidx * hdr;     // resize may move the buffer
                    uint16_t *pw = reinterpret_cast<uint16_t *>(L.recs.data() + p0);
                    for (int32_t i = 0; i < kr; ++i)
                        for (int32_t e = 0; e < 8 && gp.j0 + e < kc; ++e)
                            pw[i * 8 + e] = w[A->blk_ptr[gp.t] + (int64_t)i * kc + gp.j0 + e];
                    pay16 += (uint32_t)kr;
                }
                uint32_t *hd = reinterpret_cast<uint32_t *>(h + L.ks * 2) + g * 2;
                hd[0] = rowmask;
                hd[1] = off;
            }
            step += (int64_t)nst;
        }
        L.cptr[(size_t)ch * (A->nbr + 1) + A->nbr] = (int32_t)step;
        L.bptr[(size_t)ch * (A->nbr + 1) + A->nbr] = (int32_t)(L.recs.size() / 16);
    }
    L.nsteps = step;
    for (int gi = 0; gi < 4; ++gi) {
        const int64_t Gs = 4 << gi;
        int32_t amax = 0;
        for (int32_t ch = 0; ch < L.nchunks; ++ch) {
            const int32_t *bp = &L.bptr[(size_t)ch * (A->nbr + 1)];
            for (int64_t t0 = 0; t0 < A->nbr; t0 += Gs)
                amax = std::max(amax, bp[std::min<int64_t>(A->nbr, t0 + Gs)] - bp[t0]);
        }
        L.amax[gi] = amax;
    }
    // fits the kernel's smallest launch (strip groups of 4 << gsel)?
    return L.chunk_rows <= max_chunk_rows && (int64_t)L.amax[gsel] * 16 <= max_group_bytes && L.recs.size() < (size_t(1) << 31) * 16;
}

// max_rows: most rows of X per chunk; gsel / max_group_bytes: the records of a group of 4 << gsel strips must fit
// max_group_bytes per chunk (the kernel's LDS room for them)
void build_mma_layout(grim_bcr_matrix *A, MmaLayout &L, int32_t chunk_rows_opt, int32_t max_rows, int gsel,
                      int64_t max_group_bytes) {
    L.present = false;
    if (A->dtype == GRIM_F32) return;
    if (A->BR != 16 && A->BR != 32) return;
    if (A->BC > max_rows) return;
    const int32_t want = chunk_rows_opt > 0 ? std::min<int32_t>(chunk_rows_opt, max_rows) : max_rows;
    // largest chunk whose weight records still leave room in LDS; denser matrices get smaller chunks
    int32_t blocks = std::max<int32_t>(1, want / A->BC);
    bool fits = build_mma_layout_for(A, L, blocks, max_rows, gsel, max_group_bytes);
    while (!fits && blocks > 1) {
        blocks = (blocks + 1) / 2;
        fits = build_mma_layout_for(A, L, blocks, max_rows, gsel, max_group_bytes);
    }
    if (!fits) {   // even one column block per chunk overflows LDS: leave this matrix to the FMA kernel
        L.cptr.clear(); L.bptr.clear(); L.recs.clear();
        return;
    }
    L.present = true;
}

// ---- derived layout: row-gathering SpMM ----------------------------------------------------
void build_gather_layout(grim_bcr_matrix *A) {
    GatherLayout &L = A->gather;
    L = GatherLayout();
    // Block heights that divide 16 or are multiples of 16 map onto 16-row MFMA tiles: stored rows
    // (stored strip p, local row r) are numbered p * BR + r and cut into runs of 16.
    if (A->dtype == GRIM_F32 || A->K > 0x7fffffff || A->M > 0x7fffffff) return;
    if (!(16 % A->BR == 0 || A->BR % 16 == 0)) return;
    const uint16_t *w = reinterpret_cast<const uint16_t *>(A->weights.data());
    const int64_t nss = (A->M + 15) / 16;                 // 16-row strips of the stored order
    L.nstrips = nss;
    L.sptr.assign((size_t)nss + 1, 0);
    L.out_row.assign((size_t)nss * 16, -1);
    for (int64_t p = 0; p < A->nbr; ++p)
        for (int32_t r = 0; r < A->BR; ++r)
            L.out_row[(size_t)(p * A->BR + r)] = (int32_t)((int64_t)A->strip_order[p] * A->BR + r);
    struct Group { int64_t t; int32_t j0; uint32_t rowmask; int32_t rlo, rhi; };   // rows [rlo, rhi) of the block's kept list
    std::vector<Group> groups;
    for (int64_t u = 0; u < nss; ++u) {
        L.sptr[(size_t)u] = (int32_t)L.nsteps;
        groups.clear();
        const int64_t row0 = u * 16, row1 = std::min<int64_t>(A->M, row0 + 16);
        const int64_t p0 = row0 / A->BR, p1 = (row1 - 1) / A->BR;           // stored strips that overlap this run
        for (int64_t c = 0; c < A->nbc; ++c) {
            for (int64_t p = p0; p <= p1; ++p) {
                const int64_t t = p * A->nbc + c;
                const int32_t kr = A->row_ptr[t + 1] - A->row_ptr[t], kc = A->col_ptr[t + 1] - A->col_ptr[t];
                if (kr == 0 || kc == 0) continue;
                // the block's kept rows that fall into this run, as bits of the run's 16 rows
                uint32_t rowmask = 0;
                int32_t rlo = -1, rhi = -1;
                for (int32_t i = 0; i < kr; ++i) {
                    const int64_t sr = p * A->BR + A->row_idx[A->row_ptr[t] + i];
                    if (sr < row0 || sr >= row1) continue;
                    rowmask |= 1u << (sr - row0);
                    if (rlo < 0) rlo = i;
                    rhi = i + 1;
                }
                if (!rowmask) continue;
                for (int32_t j0 = 0; j0 < kc; j0 += 8) groups.push_back({t, j0, rowmask, rlo, rhi});
            }
        }
        while (groups.size() % 4) groups.push_back({-1, 0, 0u, 0, 0});
        const size_t nst = groups.size() / 4;
        if ((uint64_t)L.nsteps + nst > 0x7fffffffu) { L = GatherLayout(); return; }
        const size_t step0 = (size_t)L.nsteps;
        L.rows.resize((step0 + nst) * 32, 0xffffffffu);
        L.desc.resize((step0 + nst) * 8, 0u);
        for (size_t q = 0; q < groups.size(); ++q) {
            const Group &gp = groups[q];
            const size_t step = step0 + q / 4, g = q % 4;
            if (gp.t < 0) continue;                       // padding group: rows stay 0xffffffff, mask 0
            const int32_t kc = A->col_ptr[gp.t + 1] - A->col_ptr[gp.t];
            const int64_t c = gp.t % A->nbc;
            for (int32_t j = 0; j < 8 && gp.j0 + j < kc; ++j) {
                L.rows[step * 32 + (size_t)j * 4 + g] = (uint32_t)(c * A->BC + A->col_idx[A->col_ptr[gp.t] + gp.j0 + j]);
                ++L.xrows;
            }
            const int32_t nrows = gp.rhi - gp.rlo;        // kept rows are ascending, so the run's share is contiguous
            const size_t pl0 = L.payload.size();
            if (pl0 / 16 + (size_t)nrows > 0xffffffffu) { L = GatherLayout(); return; }
            L.payload.resize(pl0 + (size_t)nrows * 16, 0);
            uint16_t *pw = reinterpret_cast<uint16_t *>(L.payload.data() + pl0);
            for (int32_t i = 0; i < nrows; ++i)
                for (int32_t e = 0; e < 8 && gp.j0 + e < kc; ++e)
                    pw[i * 8 + e] = w[A->blk_ptr[gp.t] + (int64_t)(gp.rlo + i) * kc + gp.j0 + e];
            L.desc[step * 8 + g * 2] = gp.rowmask;
            L.desc[step * 8 + g * 2 + 1] = (uint32_t)(pl0 / 16);
        }
        L.nsteps += (int64_t)nst;
    }
    L.sptr[(size_t)nss] = (int32_t)L.nsteps;
    L.usteps = nss > 0 ? L.sptr[1] - L.sptr[0] : 0;
    for (int64_t u = 0; u < nss && L.usteps > 0; ++u)
        if (L.sptr[(size_t)u + 1] - L.sptr[(size_t)u] != L.usteps) L.usteps = 0;
    L.max_steps = 0;
    for (int64_t u = 0; u < nss; ++u) L.max_steps = std::max<int32_t>(L.max_steps, L.sptr[(size_t)u + 1] - L.sptr[(size_t)u]);
    L.present = true;
}

// ---- derived layout: SpMV --------------------------------------------------------------
void build_gemv_layout(grim_bcr_matrix *A) {
    GemvLayout &G = A->gemv;
    G.present = false;
    G.krmax = G.kcmax = 0;
    if (A->BR > 32 || A->BC > 32) return;
    if (A->nnz >= (int64_t(1) << 31)) return;
    G.masks.assign((size_t)A->nb * 2, 0);
    G.woff.resize((size_t)A->nb + 1);
    int32_t ukr = -2, ukc = -2;
    int32_t vec = 8;
    for (int64_t t = 0; t < A->nb; ++t) {
        uint32_t rm = 0, cm = 0;
        for (int32_t q = A->row_ptr[t]; q < A->row_ptr[t + 1]; ++q) rm |= 1u << A->row_idx[q];
        for (int32_t q = A->col_ptr[t]; q < A->col_ptr[t + 1]; ++q) cm |= 1u << A->col_idx[q];
        int32_t kr = A->row_ptr[t + 1] - A->row_ptr[t], kc = A->col_ptr[t + 1] - A->col_ptr[t];
        if (kr == 0 || kc == 0) { rm = 0; cm = 0; kr = 0; kc = 0; }   // stores nothing
        G.masks[2 * t] = rm;
        G.masks[2 * t + 1] = cm;
        G.woff[t] = (uint32_t)A->blk_ptr[t];
        ukr = ukr == -2 ? kr : (ukr == kr ? ukr : -1);
        ukc = ukc == -2 ? kc : (ukc == kc ? ukc : -1);
        if (kr > 0) while (vec > 1 && kc % vec) vec >>= 1;
        G.krmax = std::max(G.krmax, kr);
        G.kcmax = std::max(G.kcmax, kc);
    }
    G.woff[A->nb] = (uint32_t)A->blk_ptr[A->nb];
    G.uniform_kr = ukr < 0 ? -1 : ukr;
    G.uniform_kc = ukc < 0 ? -1 : ukc;
    if (G.uniform_kr < 0 || G.uniform_kc < 0) G.uniform_kr = G.uniform_kc = -1;
    G.vec = std::min<int32_t>(vec, 16 / dtype_size(A->dtype));
    G.present = true;
}

grim_status upload(grim_bcr_matrix *A) {
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) { (void)hipGetLastError(); return GRIM_ERR_DEVICE; }
    if (hipGetDevice(&A->device) != hipSuccess) return GRIM_ERR_DEVICE;
    Slab s;
    auto bytes = [](const auto &v) { return v.size() * sizeof(v[0]); };
    std::vector<int32_t> strip_pos((size_t)A->nbr);
    for (int64_t q = 0; q < A->nbr; ++q) strip_pos[(size_t)A->strip_order[q]] = (int32_t)q;
    A->order_identity = true;
    for (int64_t q = 0; q < A->nbr; ++q) A->order_identity = A->order_identity && A->strip_order[q] == q;
    size_t o_so = s.add(bytes(A->strip_order));
    size_t o_sp = s.add(bytes(strip_pos));
    size_t o_rp = s.add(bytes(A->row_ptr));
    size_t o_ri = s.add(bytes(A->row_idx));
    size_t o_cp = s.add(bytes(A->col_ptr));
    size_t o_ci = s.add(bytes(A->col_idx));
    size_t o_bp = s.add(bytes(A->blk_ptr));
    size_t o_w = s.add(A->weights.size() + 64);   // slack: vector loads may overrun a row's end
    size_t o_rm = s.add(bytes(A->rowmask64));
    size_t canon_end = s.total;
    size_t o_kp = 0, o_bp2 = 0, o_af = 0, o_gm = 0, o_go = 0;
    if (A->mma.present) {
        o_kp = s.add(bytes(A->mma.cptr));
        o_bp2 = s.add(bytes(A->mma.bptr));
        o_af = s.add(bytes(A->mma.recs) + 2048);   // slack: records are fetched in 1 KB slots
    }
    size_t o_wkp = 0, o_wbp = 0, o_waf = 0;
    if (A->mmaw.present) {
        o_wkp = s.add(bytes(A->mmaw.cptr));
        o_wbp = s.add(bytes(A->mmaw.bptr));
        o_waf = s.add(bytes(A->mmaw.recs) + 2048);
    }
    size_t o_gs = 0, o_gq = 0, o_gr = 0, o_gd = 0, o_gp = 0;
    if (A->gather.present) {
        o_gs = s.add(bytes(A->gather.sptr));
        o_gq = s.add(bytes(A->gather.out_row));
        o_gr = s.add(bytes(A->gather.rows) + 16);
        o_gd = s.add(bytes(A->gather.desc) + 16);
        o_gp = s.add(bytes(A->gather.payload) + 16);
    }
    size_t mma_end = s.total;
    if (A->gemv.present) {
        o_gm = s.add(bytes(A->gemv.masks));
        o_go = s.add(bytes(A->gemv.woff));
    }
    char *base = nullptr;
    if (hipMalloc(reinterpret_cast<void **>(&base), s.total + 256) != hipSuccess) { (void)hipGetLastError(); return GRIM_ERR_ALLOC; }
    if (hipMemset(base, 0, s.total + 256) != hipSuccess) { (void)hipFree(base); return GRIM_ERR_DEVICE; }
    auto put = [&](size_t off, const void *src, size_t n) -> bool {
        return n == 0 || hipMemcpy(base + off, src, n, hipMemcpyHostToDevice) == hipSuccess;
    };
    bool ok = put(o_so, A->strip_order.data(), bytes(A->strip_order)) && put(o_sp, strip_pos.data(), bytes(strip_pos)) && put(o_rp, A->row_ptr.data(), bytes(A->row_ptr)) &&
              put(o_ri, A->row_idx.data(), bytes(A->row_idx)) && put(o_cp, A->col_ptr.data(), bytes(A->col_ptr)) &&
              put(o_ci, A->col_idx.data(), bytes(A->col_idx)) && put(o_bp, A->blk_ptr.data(), bytes(A->blk_ptr)) &&
              put(o_w, A->weights.data(), A->weights.size()) && put(o_rm, A->rowmask64.data(), bytes(A->rowmask64));
    if (ok && A->mma.present)
        ok = put(o_kp, A->mma.cptr.data(), bytes(A->mma.cptr)) && put(o_bp2, A->mma.bptr.data(), bytes(A->mma.bptr)) &&
             put(o_af, A->mma.recs.data(), bytes(A->mma.recs));
    if (ok && A->mmaw.present)
        ok = put(o_wkp, A->mmaw.cptr.data(), bytes(A->mmaw.cptr)) && put(o_wbp, A->mmaw.bptr.data(), bytes(A->mmaw.bptr)) &&
             put(o_waf, A->mmaw.recs.data(), bytes(A->mmaw.recs));
    if (ok && A->gather.present)
        ok = put(o_gs, A->gather.sptr.data(), bytes(A->gather.sptr)) && put(o_gq, A->gather.out_row.data(), bytes(A->gather.out_row)) && put(o_gr, A->gather.rows.data(), bytes(A->gather.rows)) &&
             put(o_gd, A->gather.desc.data(), bytes(A->gather.desc)) && put(o_gp, A->gather.payload.data(), bytes(A->gather.payload));
    if (ok && A->gemv.present)
        ok = put(o_gm, A->gemv.masks.data(), bytes(A->gemv.masks)) && put(o_go, A->gemv.woff.data(), bytes(A->gemv.woff));
    if (!ok) { (void)hipGetLastError(); (void)hipFree(base); return GRIM_ERR_DEVICE; }
    A->dev.strip_order = reinterpret_cast<int32_t *>(base + o_so);
    A->dev.strip_pos = reinterpret_cast<int32_t *>(base + o_sp);
    A->dev.row_ptr = reinterpret_cast<int32_t *>(base + o_rp);
    A->dev.row_idx = reinterpret_cast<uint16_t *>(base + o_ri);
    A->dev.col_ptr = reinterpret_cast<int32_t *>(base + o_cp);
    A->dev.col_idx = reinterpret_cast<uint16_t *>(base + o_ci);
    A->dev.blk_ptr = reinterpret_cast<int64_t *>(base + o_bp);
    A->dev.weights = base + o_w;
    A->dev.rowmask64 = reinterpret_cast<uint64_t *>(base + o_rm);
    A->dev.bytes = (int64_t)canon_end;
    if (A->mma.present) {
        A->mma.d_cptr = reinterpret_cast<int32_t *>(base + o_kp);
        A->mma.d_bptr = reinterpret_cast<int32_t *>(base + o_bp2);
        A->mma.d_recs = reinterpret_cast<unsigned char *>(base + o_af);
        A->mma.bytes = (int64_t)(mma_end - canon_end);
    }
    if (A->mmaw.present) {
        A->mmaw.d_cptr = reinterpret_cast<int32_t *>(base + o_wkp);
        A->mmaw.d_bptr = reinterpret_cast<int32_t *>(base + o_wbp);
        A->mmaw.d_recs = reinterpret_cast<unsigned char *>(base + o_waf);
        A->mmaw.bytes = (int64_t)(bytes(A->mmaw.cptr) + bytes(A->mmaw.bptr) + bytes(A->mmaw.recs));
    }
    if (A->gather.present) {
        A->gather.d_sptr = reinterpret_cast<int32_t *>(base + o_gs);
        A->gather.d_out_row = reinterpret_cast<int32_t *>(base + o_gq);
        A->gather.d_rows = reinterpret_cast<uint32_t *>(base + o_gr);
        A->gather.d_desc = reinterpret_cast<uint32_t *>(base + o_gd);
        A->gather.d_payload = reinterpret_cast<unsigned char *>(base + o_gp);
        A->gather.bytes = (int64_t)(o_gp + bytes(A->gather.payload) + 16 - o_gs);
    }
    if (A->gemv.present) {
        A->gemv.d_masks = reinterpret_cast<uint32_t *>(base + o_gm);
        A->gemv.d_woff = reinterpret_cast<uint32_t *>(base + o_go);
        A->gemv.bytes = (int64_t)(s.total - mma_end);
    }
    A->on_device = true;
    return GRIM_OK;
}

grim_status check_call(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, const float *Y, int64_t ldy) {
    if (!A || !X || !Y) return GRIM_ERR_NULL;
    if (N < 1 || ldx < N || ldy < N) return GRIM_ERR_SHAPE;
    if (N > (int64_t(1) << 30) || ldx > (int64_t(1) << 40) || ldy > (int64_t(1) << 40)) return GRIM_ERR_SHAPE;
    if (!A->on_device) return GRIM_ERR_DEVICE;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != A->device) return GRIM_ERR_DEVICE;
    return GRIM_OK;
}

bool gemv_ok(const grim_bcr_matrix *A, int64_t N) {
    return A->gemv.present && N >= 1 && N <= 8 && A->K * N * dtype_size(A->dtype) <= kGemvMaxXBytes;
}

// do the byte ranges [a, a + na) and [b, b + nb) overlap?
bool ranges_overlap(const void *a, int64_t na, const void *b, int64_t nb) {
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + (uintptr_t)nb && b0 < a0 + (uintptr_t)na;
}

GemvDesc desc_of(const grim_bcr_matrix *A) {
    return GemvDesc{A->dev.weights, A->gemv.d_masks, A->gemv.d_woff, A->dev.strip_order};
}

}  // namespace

extern "C" {

grim_status grim_bcr_pack(const void *W_host, grim_dtype dt, int64_t M, int64_t K, int64_t ldw, int32_t BR, int32_t BC,
                          const int32_t *row_ptr, const uint16_t *row_idx, const int32_t *col_ptr,
                          const uint16_t *col_idx, const grim_bcr_options *opt, grim_bcr_matrix **out) {
    if (out) *out = nullptr;
    if (!out || !W_host || !row_ptr || !col_ptr) return GRIM_ERR_NULL;
    if (dt != GRIM_F32 && dt != GRIM_F16 && dt != GRIM_BF16) return GRIM_ERR_DTYPE;
    if (M < 1 || K < 1 || BR < 1 || BC < 1 || BR > 65535 || BC > 65535) return GRIM_ERR_SHAPE;
    if (M % BR || K % BC || ldw < K) return GRIM_ERR_SHAPE;
    if (M > (int64_t(1) << 31) - 1 || K > (int64_t(1) << 31) - 1) return GRIM_ERR_SHAPE;
    const int64_t nbr = M / BR, nbc = K / BC;
    if (nbr > (int64_t(1) << 30) / nbc) return GRIM_ERR_SHAPE;   // ptr arrays are 32-bit
    const int64_t nb = nbr * nbc;
    grim_status st = validate_sets(nb, BR, row_ptr, row_idx);
    if (st != GRIM_OK) return st;
    st = validate_sets(nb, BC, col_ptr, col_idx);
    if (st != GRIM_OK) return st;

    grim_bcr_matrix *A = nullptr;
    try {
        A = new grim_bcr_matrix();
        A->M = M; A->K = K; A->BR = BR; A->BC = BC; A->dtype = dt;
        A->nbr = nbr; A->nbc = nbc; A->nb = nb;
        A->reordered = !(opt && opt->no_reorder);
        // strip work = stored weights of the strip; heavier strips first, ties by index (Section 4.2)
        std::vector<int64_t> work(nbr, 0);
        for (int64_t s = 0; s < nbr; ++s)
            for (int64_t c = 0; c < nbc; ++c) {
                int64_t b = s * nbc + c;
                work[s] += int64_t(row_ptr[b + 1] - row_ptr[b]) * int64_t(col_ptr[b + 1] - col_ptr[b]);
            }
        A->strip_order.resize(nbr);
        std::iota(A->strip_order.begin(), A->strip_order.end(), 0);
        if (A->reordered)
            std::stable_sort(A->strip_order.begin(), A->strip_order.end(),
                             [&](int32_t a, int32_t b) { return work[a] > work[b]; });
        const int esz = dtype_size(dt);
        A->row_ptr.assign(nb + 1, 0);
        A->col_ptr.assign(nb + 1, 0);
        A->blk_ptr.assign(nb + 1, 0);
        A->rowmask64.assign(nb, 0);
        int64_t t = 0;
        for (int64_t p = 0; p < nbr; ++p) {
            int64_t s = A->strip_order[p];
            for (int64_t c = 0; c < nbc; ++c, ++t) {
                int64_t b = s * nbc + c;
                int32_t kr = row_ptr[b + 1] - row_ptr[b], kc = col_ptr[b + 1] - col_ptr[b];
                A->row_ptr[t + 1] = A->row_ptr[t] + kr;
                A->col_ptr[t + 1] = A->col_ptr[t] + kc;
                A->blk_ptr[t + 1] = A->blk_ptr[t] + int64_t(kr) * kc;
            }
        }
        A->nnz = A->blk_ptr[nb];
        A->row_idx.resize(A->row_ptr[nb]);
        A->col_idx.resize(A->col_ptr[nb]);
        A->weights.resize((size_t)A->nnz * esz);
        const unsigned char *W = static_cast<const unsigned char *>(W_host);
        t = 0;
        for (int64_t p = 0; p < nbr; ++p) {
            int64_t s = A->strip_order[p];
            for (int64_t c = 0; c < nbc; ++c, ++t) {
                int64_t b = s * nbc + c;
                int32_t kr = row_ptr[b + 1] - row_ptr[b], kc = col_ptr[b + 1] - col_ptr[b];
                const uint16_t *R = kr ? row_idx + row_ptr[b] : nullptr;
                const uint16_t *C = kc ? col_idx + col_ptr[b] : nullptr;
                for (int32_t i = 0; i < kr; ++i) {
                    A->row_idx[A->row_ptr[t] + i] = R[i];
                    if (BR <= 64) A->rowmask64[t] |= uint64_t(1) << R[i];
                }
                for (int32_t j = 0; j < kc; ++j) A->col_idx[A->col_ptr[t] + j] = C[j];
                unsigned char *dst = A->weights.data() + (size_t)A->blk_ptr[t] * esz;
                for (int32_t i = 0; i < kr; ++i) {
                    const unsigned char *src = W + ((s * BR + R[i]) * ldw + c * BC) * esz;
                    for (int32_t j = 0; j < kc; ++j) std::memcpy(dst + ((size_t)i * kc + j) * esz, src + (size_t)C[j] * esz, esz);
                }
            }
        }
        if (!(opt && opt->host_only == 1)) {
            // staged kernel: chunks of up to 256 rows, a 4-strip group's records within 16 KB (the producers move at
            // most 32 KB of X rows and 16 KB of records per chunk); wide-tile kernel: chunks of up to 128 or 192 rows, a
            // 16-strip group's records within 32 KB
            build_mma_layout(A, A->mma, opt ? opt->chunk_rows : 0, kMmaMaxChunkRows, 0, 16 * 1024);
            build_mma_layout(A, A->mmaw, opt ? opt->chunk_rows : 0, wide_max_chunk_rows(A->BR), 2, kWideMaxRecordBytes);
            build_gather_layout(A);
            build_gemv_layout(A);
        }
    } catch (const std::bad_alloc &) {
        delete A;
        return GRIM_ERR_ALLOC;
    }
    if (!(opt && opt->host_only)) {
        st = upload(A);
        if (st != GRIM_OK) { delete A; return st; }
    }
    *out = A;
    return GRIM_OK;
}

grim_status grim_bcr_unpack(const grim_bcr_matrix *A, void *W_host_out, int64_t ldw) {
    if (!A || !W_host_out) return GRIM_ERR_NULL;
    if (ldw < A->K) return GRIM_ERR_SHAPE;
    const int esz = dtype_size(A->dtype);
    unsigned char *W = static_cast<unsigned char *>(W_host_out);
    for (int64_t i = 0; i < A->M; ++i) std::memset(W + i * ldw * esz, 0, (size_t)A->K * esz);
    int64_t t = 0;
    for (int64_t p = 0; p < A->nbr; ++p) {
        int64_t s = A->strip_order[p];
        for (int64_t c = 0; c < A->nbc; ++c, ++t) {
            int32_t kr = A->row_ptr[t + 1] - A->row_ptr[t], kc = A->col_ptr[t + 1] - A->col_ptr[t];
            const unsigned char *src = A->weights.data() + (size_t)A->blk_ptr[t] * esz;
            for (int32_t i = 0; i < kr; ++i) {
                int64_t r = s * A->BR + A->row_idx[A->row_ptr[t] + i];
                for (int32_t j = 0; j < kc; ++j) {
                    int64_t k = c * A->BC + A->col_idx[A->col_ptr[t] + j];
                    std::memcpy(W + (r * ldw + k) * esz, src + ((size_t)i * kc + j) * esz, esz);
                }
            }
        }
    }
    return GRIM_OK;
}

grim_status grim_bcr_unpack_layout(const grim_bcr_matrix *A, int32_t layout, void *W_host_out, int64_t ldw) {
    if (!A || !W_host_out) return GRIM_ERR_NULL;
    if (ldw < A->K) return GRIM_ERR_SHAPE;
    const int esz = dtype_size(A->dtype);
    unsigned char *W = static_cast<unsigned char *>(W_host_out);
    auto clear = [&]() { for (int64_t i = 0; i < A->M; ++i) std::memset(W + i * ldw * esz, 0, (size_t)A->K * esz); };
    auto put = [&](int64_t r, int64_t k, const void *src) { std::memcpy(W + (r * ldw + k) * esz, src, esz); };
    if (layout == 1 || layout == 4) {
        // staged matrix-core layouts: regions of [steps x header][payload] per (chunk, stored strip)
        const MmaLayout &L = layout == 1 ? A->mma : A->mmaw;
        if (!L.present) return GRIM_ERR_UNSUPPORTED;
        clear();
        const int32_t ng = L.ks / 8, hdr = L.ks * 2 + ng * 8;
        for (int32_t ch = 0; ch < L.nchunks; ++ch) {
            for (int64_t st = 0; st < A->nbr; ++st) {
                const size_t e = (size_t)ch * (A->nbr + 1) + st;
                const int32_t nst = L.cptr[e + 1] - L.cptr[e];
                const unsigned char *region = L.recs.data() + (size_t)L.bptr[e] * 16;
                for (int32_t s = 0; s < nst; ++s) {
                    const unsigned char *h = region + (size_t)s * hdr;
                    for (int32_t g = 0; g < ng; ++g) {
                        const uint16_t *hs = reinterpret_cast<const uint16_t *>(h) + g * 8;
                        const uint32_t *hd = reinterpret_cast<const uint32_t *>(h + L.ks * 2) + g * 2;
                        const uint32_t rowmask = hd[0];
                        const unsigned char *pw = region + (size_t)hd[1] * 16;
                        int32_t i = 0;
                        for (int32_t r = 0; r < A->BR; ++r) {
                            if (!((rowmask >> r) & 1u)) continue;
                            for (int32_t slot = 0; slot < 8; ++slot) {
                                const uint16_t srow = slot < 4 ? hs[2 * slot] : hs[2 * (slot - 4) + 1];
                                if (srow == (uint16_t)L.chunk_rows) continue;      // the zero row: padding
                                put((int64_t)A->strip_order[st] * A->BR + r, (int64_t)ch * L.chunk_rows + srow,
                                    pw + ((size_t)i * 8 + slot) * 2);
                            }
                            ++i;
                        }
                    }
                }
            }
        }
        return GRIM_OK;
    }
    if (layout == 2) {
        // row-gathering layout: per 16-row run a list of steps of four groups of 8 k slots
        const GatherLayout &L = A->gather;
        if (!L.present) return GRIM_ERR_UNSUPPORTED;
        clear();
        for (int64_t u = 0; u < L.nstrips; ++u) {
            for (int64_t s = L.sptr[(size_t)u]; s < L.sptr[(size_t)u + 1]; ++s) {
                for (int32_t g = 0; g < 4; ++g) {
                    const uint32_t rowmask = L.desc[(size_t)s * 8 + g * 2];
                    const unsigned char *pw = L.payload.data() + (size_t)L.desc[(size_t)s * 8 + g * 2 + 1] * 16;
                    int32_t i = 0;
                    for (int32_t r = 0; r < 16; ++r) {
                        if (!((rowmask >> r) & 1u)) continue;
                        const int32_t orow = L.out_row[(size_t)u * 16 + r];
                        for (int32_t j = 0; j < 8; ++j) {
                            const uint32_t k = L.rows[(size_t)s * 32 + (size_t)j * 4 + g];
                            if (k == 0xffffffffu) continue;
                            if (orow < 0 || k >= (uint32_t)A->K) return GRIM_ERR_INDEX;
                            put(orow, k, pw + ((size_t)i * 8 + j) * 2);
                        }
                        ++i;
                    }
                }
            }
        }
        return GRIM_OK;
    }
    if (layout == 3) {
        // SpMV layout: the compact weights with one row and one column bit mask per stored block
        const GemvLayout &G = A->gemv;
        if (!G.present) return GRIM_ERR_UNSUPPORTED;
        clear();
        for (int64_t t = 0; t < A->nb; ++t) {
            const uint32_t rm = G.masks[2 * (size_t)t], cm = G.masks[2 * (size_t)t + 1];
            const int32_t kc = __builtin_popcount(cm);
            const int64_t p = t / A->nbc, c = t % A->nbc;
            int32_t i = 0;
            for (int32_t r = 0; r < A->BR; ++r) {
                if (!((rm >> r) & 1u)) continue;
                int32_t j = 0;
                for (int32_t q = 0; q < A->BC; ++q) {
                    if (!((cm >> q) & 1u)) continue;
                    put((int64_t)A->strip_order[p] * A->BR + r, c * A->BC + q,
                        A->weights.data() + ((size_t)G.woff[(size_t)t] + (size_t)i * kc + j) * esz);
                    ++j;
                }
                ++i;
            }
        }
        return GRIM_OK;
    }
    return GRIM_ERR_SHAPE;
}

grim_status grim_bcr_export_bcrc(const grim_bcr_matrix *A, grim_bcrc **out) {
    if (out) *out = nullptr;
    if (!A || !out) return GRIM_ERR_NULL;
    if (A->M > 0x7fffffff || A->K > 0x7fffffff) return GRIM_ERR_SHAPE;
    grim_bcrc *B = nullptr;
    try {
        B = new grim_bcrc();
        B->M = A->M; B->K = A->K; B->dtype = A->dtype;
        const int esz = dtype_size(A->dtype);
        // stored position of every strip
        std::vector<int64_t> pos((size_t)A->nbr);
        for (int64_t p = 0; p < A->nbr; ++p) pos[(size_t)A->strip_order[p]] = p;
        // per original row: its kept global columns, and where each block's run of weights starts
        struct Run { int64_t w0; int32_t kc; };
        std::vector<std::vector<int32_t>> pattern((size_t)A->M);
        std::vector<std::vector<Run>> runs((size_t)A->M);
        for (int64_t s = 0; s < A->nbr; ++s) {
            for (int64_t c = 0; c < A->nbc; ++c) {
                const int64_t t = pos[(size_t)s] * A->nbc + c;
                const int32_t kr = A->row_ptr[t + 1] - A->row_ptr[t], kc = A->col_ptr[t + 1] - A->col_ptr[t];
                if (!kr || !kc) continue;
                for (int32_t i = 0; i < kr; ++i) {
                    const int64_t r = s * A->BR + A->row_idx[A->row_ptr[t] + i];
                    for (int32_t j = 0; j < kc; ++j)
                        pattern[(size_t)r].push_back((int32_t)(c * A->BC + A->col_idx[A->col_ptr[t] + j]));
                    runs[(size_t)r].push_back({A->blk_ptr[t] + (int64_t)i * kc, kc});
                }
            }
        }
        // groups in order of first appearance
        std::map<std::vector<int32_t>, int32_t> ids;
        std::vector<std::vector<int32_t>> members;
        for (int64_t r = 0; r < A->M; ++r) {
            auto it = ids.find(pattern[(size_t)r]);
            if (it == ids.end()) {
                it = ids.emplace(pattern[(size_t)r], (int32_t)members.size()).first;
                members.emplace_back();
            }
            members[(size_t)it->second].push_back((int32_t)r);
        }
        B->occurrence.push_back(0);
        B->column_stride.push_back(0);
        B->row_offset.push_back(0);
        B->weights.reserve(A->weights.size());
        for (const auto &grp : members) {
            const std::vector<int32_t> &cols = pattern[(size_t)grp[0]];
            B->compact_column.insert(B->compact_column.end(), cols.begin(), cols.end());
            B->column_stride.push_back((int64_t)B->compact_column.size());
            for (int32_t r : grp) {
                B->reorder.push_back(r);
                for (const Run &run : runs[(size_t)r]) {
                    const unsigned char *src = A->weights.data() + (size_t)run.w0 * esz;
                    B->weights.insert(B->weights.end(), src, src + (size_t)run.kc * esz);
                }
                B->row_offset.push_back((int64_t)(B->weights.size() / esz));
            }
            B->occurrence.push_back((int32_t)B->reorder.size());
        }
    } catch (const std::bad_alloc &) {
        delete B;
        return GRIM_ERR_ALLOC;
    }
    *out = B;
    return GRIM_OK;
}

grim_status grim_bcrc_arrays(const grim_bcrc *B, grim_bcrc_view *v) {
    if (!B || !v) return GRIM_ERR_NULL;
    v->M = B->M; v->K = B->K; v->dtype = B->dtype;
    v->ngroups = (int64_t)B->occurrence.size() - 1;
    v->nnz = B->row_offset.back();
    v->ncols = (int64_t)B->compact_column.size();
    v->reorder = B->reorder.data();
    v->row_offset = B->row_offset.data();
    v->occurrence = B->occurrence.data();
    v->column_stride = B->column_stride.data();
    v->compact_column = B->compact_column.data();
    v->weights = B->weights.data();
    return GRIM_OK;
}

void grim_bcrc_free(grim_bcrc *B) { delete B; }

grim_status grim_bcr_arrays(const grim_bcr_matrix *A, grim_bcr_view *v) {
    if (!A || !v) return GRIM_ERR_NULL;
    v->M = A->M; v->K = A->K; v->BR = A->BR; v->BC = A->BC; v->dtype = A->dtype; v->reordered = A->reordered;
    v->nbr = A->nbr; v->nbc = A->nbc; v->nb = A->nb; v->nnz = A->nnz;
    v->strip_order = A->strip_order.data();
    v->row_ptr = A->row_ptr.data();
    v->row_idx = A->row_idx.data();
    v->col_ptr = A->col_ptr.data();
    v->col_idx = A->col_idx.data();
    v->blk_ptr = A->blk_ptr.data();
    v->weights = A->weights.data();
    v->dev_bytes_canonical = A->on_device ? A->dev.bytes : 0;
    v->dev_bytes_mma = A->on_device && A->mma.present ? A->mma.bytes : 0;
    v->dev_bytes_gemv = A->on_device && A->gemv.present ? A->gemv.bytes : 0;
    return GRIM_OK;
}

// Eight right-hand sides in 16-byte-aligned rows: one (padded) tile of the row-gathering matrix-core
// kernel beats the vector-ALU SpMV kernel (4096 x 2048 at 10.7x: 8.0 -> 5.6 us; at 4 it does not)
// a few columns of a uniformly pruned matrix: the one-column SpMV kernel on a set of workgroups per column, while all
// sets fit the GPU in one round
// (`count`: products of this shape in the launch -- 2 for the two sides of a GRU step)
static bool columns_as_sets(const grim_bcr_matrix *A, int64_t N, int count) {
    return N > 1 && N <= 8 && gemv_ok(A, N) && A->BR <= 32 && A->BC <= 32 &&
           spmv_exact_applies(A->dtype, A->gemv.uniform_kr, A->gemv.uniform_kc, A->K) &&
           spmv_column_sets_ok(count, A->nbr, (int32_t)N);
}

static bool skinny_on_matrix_cores(const grim_bcr_matrix *A, const void *X_dev, int64_t N, int64_t ldx, int count = 1) {
    return N == 8 && !columns_as_sets(A, N, count) && ldx % 8 == 0 && reinterpret_cast<uintptr_t>(X_dev) % 16 == 0 &&
           gather_applies(A, X_dev, N, ldx);
}

// which kernel family a grim_bcr_spmm_tuned call runs
enum SpmmRoute { ROUTE_NONE, ROUTE_SPMV, ROUTE_FMA, ROUTE_MMA, ROUTE_GATHER, ROUTE_WIDE };

// what the columns the wide-tile kernel leaves over cost on the kernels that take any N
static double rest_cost(const grim_bcr_matrix *A, int64_t n) {
    int tn = 0, g = 0;
    double best = A->mma.present ? mma_best_shape(A, n, 0, 0, &tn, &g) : -1.0;
    if (A->gather.present && n % 4 == 0) {
        const double c = gather_cost(A, n);
        if (best < 0 || c < best) best = c;
    }
    return best;
}

// `wide_tn` / `wide_cols`: for ROUTE_WIDE, the tile width and the leading columns that kernel takes
static SpmmRoute spmm_route(const grim_bcr_matrix *A, const void *X_dev, int64_t N, int64_t ldx, const float *Y_dev,
                            int64_t ldy, int32_t tile_n, int32_t strips_per_wg, int32_t kernel, int *wide_tn,
                            int64_t *wide_cols) {
    if (kernel < 0 || kernel > 4 || tile_n < 0 || strips_per_wg < 0) return ROUTE_NONE;
    const bool free_choice = kernel == 0 && tile_n == 0 && strips_per_wg == 0;
    if (kernel == 3) return !tile_n && !strips_per_wg && gather_applies(A, X_dev, N, ldx) ? ROUTE_GATHER : ROUTE_NONE;
    if (kernel == 4) {
        *wide_tn = tile_n;
        *wide_cols = N;
        return !strips_per_wg && wide_applies(A, X_dev, N, ldx, Y_dev, ldy, tile_n) ? ROUTE_WIDE : ROUTE_NONE;
    }
    if (free_choice && skinny_on_matrix_cores(A, X_dev, N, ldx)) return ROUTE_GATHER;
    if (free_choice && gemv_ok(A, N)) return ROUTE_SPMV;
    const bool mma = A->mma.present && kernel != 1;
    if (kernel == 2 && !mma) return ROUTE_NONE;
    if (free_choice) {
        // the matrix-core kernels that apply: take the one that moves fewer bytes through a compute unit
        int tn = 0, g = 0;
        const double staged = mma ? mma_best_shape(A, N, 0, 0, &tn, &g) : -1.0;
        const double gather = gather_applies(A, X_dev, N, ldx) ? gather_cost(A, N) : -1.0;
        const double wide = wide_plan(A, X_dev, N, ldx, Y_dev, ldy, rest_cost, wide_tn, wide_cols);
        if (wide >= 0 && (staged < 0 || wide < staged) && (gather < 0 || wide < gather)) return ROUTE_WIDE;
        if (gather >= 0 && (staged < 0 || gather < staged)) return ROUTE_GATHER;
    }
    if (mma) return ROUTE_MMA;
    return A->BR > 64 ? ROUTE_NONE : ROUTE_FMA;
}

grim_status grim_bcr_spmm_tuned(const grim_bcr_matrix *A, const void *X_dev, int64_t N, int64_t ldx, float *Y_dev,
                                int64_t ldy, int32_t tile_n, int32_t strips_per_wg, int32_t kernel, void *hip_stream) {
    grim_status st = check_call(A, X_dev, N, ldx, Y_dev, ldy);
    if (st != GRIM_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int wide_tn = 0;
    int64_t wide_cols = 0;
    switch (spmm_route(A, X_dev, N, ldx, Y_dev, ldy, tile_n, strips_per_wg, kernel, &wide_tn, &wide_cols)) {
        case ROUTE_SPMV: {
            GemvDesc d = desc_of(A);
            return launch_spmv(nullptr, d, nullptr, 1, A->M, A->K, A->BR, A->BC, A->dtype, A->gemv.uniform_kr, A->gemv.uniform_kc,
                               A->gemv.vec, A->gemv.krmax, A->gemv.kcmax, X_dev, 0, (int32_t)N, ldx, Y_dev, 0, ldy, stream);
        }
        case ROUTE_GATHER: return launch_spmm_gather(A, X_dev, N, ldx, Y_dev, ldy, stream);
        case ROUTE_WIDE: {
            // whole rounds of fat workgroups, the few columns left over on whatever suits them: in the same launch when
            // that is the row-gathering kernel in the form the combined kernel carries, else in a launch of their own
            const char *x_rest = static_cast<const char *>(X_dev) + wide_cols * dtype_size(A->dtype);
            if (wide_cols < N) {
                int tn2 = 0;
                int64_t cols2 = 0;
                if (spmm_route(A, x_rest, N - wide_cols, ldx, Y_dev + wide_cols, ldy, 0, 0, 0, &tn2, &cols2) == ROUTE_GATHER) {
                    st = launch_spmm_wide_with_rest(A, X_dev, N, ldx, Y_dev, ldy, wide_tn, wide_cols, stream);
                    if (st != GRIM_ERR_UNSUPPORTED) return st;
                }
            }
            st = launch_spmm_wide(A, X_dev, wide_cols, ldx, Y_dev, ldy, wide_tn, stream);
            if (st != GRIM_OK || wide_cols >= N) return st;
            return grim_bcr_spmm_tuned(A, x_rest, N - wide_cols, ldx, Y_dev + wide_cols, ldy, 0, 0, 0, hip_stream);
        }
        case ROUTE_MMA: {
            if (kernel == 0 && tile_n == 0 && strips_per_wg == 0) {
                // whole rounds of workgroups on the staged kernel, the few columns left over on whatever suits them
                int tn = 0, g = 0;
                // (whether the rest may take the row-gathering kernel hangs on N and the alignment of X alone: the cut
                // is a multiple of 32 columns)
                const int64_t n_main = mma_whole_rounds(A, N, gather_applies(A, X_dev, N, ldx), &tn, &g);
                if (n_main < N) {
                    st = launch_spmm_mma(A, X_dev, n_main, ldx, Y_dev, ldy, tn, g, stream);
                    if (st != GRIM_OK) return st;
                    const char *x_rest = static_cast<const char *>(X_dev) + n_main * dtype_size(A->dtype);
                    return grim_bcr_spmm_tuned(A, x_rest, N - n_main, ldx, Y_dev + n_main, ldy, 0, 0, 0, hip_stream);
                }
            }
            return launch_spmm_mma(A, X_dev, N, ldx, Y_dev, ldy, tile_n, strips_per_wg, stream);
        }
        case ROUTE_FMA: return launch_spmm_fma(A, X_dev, N, ldx, Y_dev, ldy, stream);
        case ROUTE_NONE: break;
    }
    return GRIM_ERR_UNSUPPORTED;
}

const char *grim_bcr_spmm_kernel_name(const grim_bcr_matrix *A, const void *X_dev, int64_t N, int64_t ldx, int32_t tile_n,
                                      int32_t strips_per_wg, int32_t kernel) {
    if (!A || !X_dev || N < 1 || ldx < N || !A->on_device) return "none";
    // (the output is taken to be 16-byte aligned with a leading dimension of N rounded up to 4, as allocators give it)
    int wide_tn = 0;
    int64_t wide_cols = 0;
    switch (spmm_route(A, X_dev, N, ldx, reinterpret_cast<const float *>(uintptr_t(256)), (N + 3) / 4 * 4, tile_n, strips_per_wg,
                       kernel, &wide_tn, &wide_cols)) {
        case ROUTE_SPMV: return "bcr_spmv";
        case ROUTE_WIDE: return "bcr_spmm_wide";
        case ROUTE_GATHER: return "bcr_spmm_gather";
        case ROUTE_MMA: return "bcr_spmm_mma";
        case ROUTE_FMA: return "bcr_spmm_fma";
        case ROUTE_NONE: break;
    }
    return "none";
}

grim_status grim_bcr_spmm(const grim_bcr_matrix *A, const void *X_dev, int64_t N, int64_t ldx, float *Y_dev, int64_t ldy,
                          void *hip_stream) {
    return grim_bcr_spmm_tuned(A, X_dev, N, ldx, Y_dev, ldy, 0, 0, 0, hip_stream);
}

grim_status grim_bcr_spmv(const grim_bcr_matrix *A, const void *x_dev, int32_t batch, int64_t ldx, float *y_dev,
                          int64_t ldy, void *hip_stream) {
    if (!A || !x_dev || !y_dev) return GRIM_ERR_NULL;
    if (batch < 1 || batch > 8) return GRIM_ERR_SHAPE;
    grim_status st = check_call(A, x_dev, batch, ldx, y_dev, ldy);
    if (st != GRIM_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (skinny_on_matrix_cores(A, x_dev, batch, ldx)) return launch_spmm_gather(A, x_dev, batch, ldx, y_dev, ldy, stream);
    if (gemv_ok(A, batch)) {
        GemvDesc d = desc_of(A);
        return launch_spmv(nullptr, d, nullptr, 1, A->M, A->K, A->BR, A->BC, A->dtype, A->gemv.uniform_kr, A->gemv.uniform_kc,
                           A->gemv.vec, A->gemv.krmax, A->gemv.kcmax, x_dev, 0, batch, ldx, y_dev, 0, ldy, stream);
    }
    // blocks the SpMV kernels do not take (more than 32 rows or columns): whatever the SpMM entry point picks
    return grim_bcr_spmm_tuned(A, x_dev, batch, ldx, y_dev, ldy, 0, 0, 0, hip_stream);
}

static grim_status conv_call(const grim_bcr_matrix *A, const void *F_dev, int32_t Cin, int32_t H, int32_t W, int32_t kh,
                             int32_t kw, const float *bias_dev, int32_t relu, void *out_dev, int32_t odt, int64_t ldo,
                             void *hip_stream) {
    if (!A || !F_dev || !out_dev) return GRIM_ERR_NULL;
    if (Cin < 1 || H < 1 || W < 1 || kh < 1 || kw < 1 || kh % 2 == 0 || kw % 2 == 0) return GRIM_ERR_SHAPE;
    if ((int64_t)Cin * kh * kw != A->K || ldo < (int64_t)H * W) return GRIM_ERR_SHAPE;
    if (odt != GRIM_F32 && odt != GRIM_F16 && odt != GRIM_BF16) return GRIM_ERR_DTYPE;
    if (!A->on_device) return GRIM_ERR_DEVICE;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != A->device) { (void)hipGetLastError(); return GRIM_ERR_DEVICE; }
    grim_status st = launch_conv_wide(A, F_dev, Cin, H, W, kh, kw, 1, 0, bias_dev, relu ? 1 : 0, out_dev, odt, ldo, 0,
                                      static_cast<hipStream_t>(hip_stream));
    if (st != GRIM_ERR_UNSUPPORTED) return st;
    return launch_conv_gather(A, F_dev, Cin, H, W, kh, kw, bias_dev, relu ? 1 : 0, out_dev, odt, ldo,
                              static_cast<hipStream_t>(hip_stream));
}

grim_status grim_bcr_conv2d(const grim_bcr_matrix *A, const void *F_dev, int32_t Cin, int32_t H, int32_t W, int32_t kh,
                            int32_t kw, float *Y_dev, int64_t ldy, void *hip_stream) {
    return conv_call(A, F_dev, Cin, H, W, kh, kw, nullptr, 0, Y_dev, GRIM_F32, ldy, hip_stream);
}

grim_status grim_bcr_conv2d_act(const grim_bcr_matrix *A, const void *F_dev, int32_t Cin, int32_t H, int32_t W, int32_t kh,
                                int32_t kw, const float *bias_dev, int32_t relu, void *out_dev, grim_dtype out_dt,
                                int64_t ldo, void *hip_stream) {
    return conv_call(A, F_dev, Cin, H, W, kh, kw, bias_dev, relu, out_dev, (int32_t)out_dt, ldo, hip_stream);
}

struct grim_bcr_conv_plan {
    const grim_bcr_matrix *A = nullptr;
    int32_t Cin = 0, H = 0, W = 0, kh = 0, kw = 0, stride = 1;
    int device = -1;
    uint32_t *d_words = nullptr;
};

grim_status grim_bcr_conv_plan_create(const grim_bcr_matrix *A, int32_t Cin, int32_t H, int32_t W, int32_t kh, int32_t kw,
                                      int32_t stride, grim_bcr_conv_plan **out) {
    if (!A || !out) return GRIM_ERR_NULL;
    *out = nullptr;
    if (Cin < 1 || H < 1 || W < 1 || kh < 1 || kw < 1 || kh % 2 == 0 || kw % 2 == 0) return GRIM_ERR_SHAPE;
    if ((int64_t)Cin * kh * kw != A->K || (stride != 1 && stride != 2)) return GRIM_ERR_SHAPE;
    if (!A->on_device) return GRIM_ERR_DEVICE;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != A->device) { (void)hipGetLastError(); return GRIM_ERR_DEVICE; }
    if (!A->gather.present || kh * kw > 31 || (int64_t)Cin * H * W > (int64_t(1) << 26) || A->gather.rows.empty())
        return GRIM_ERR_UNSUPPORTED;
    std::vector<uint32_t> words(A->gather.rows.size());
    for (size_t i = 0; i < words.size(); ++i) words[i] = conv_plan_word(A->gather.rows[i], H, W, kh, kw);
    std::unique_ptr<grim_bcr_conv_plan> P(new (std::nothrow) grim_bcr_conv_plan);
    if (!P) return GRIM_ERR_ALLOC;
    P->A = A; P->Cin = Cin; P->H = H; P->W = W; P->kh = kh; P->kw = kw; P->stride = stride; P->device = dev;
    void *ptr = nullptr;
    if (hipMalloc(&ptr, words.size() * 4) != hipSuccess) { (void)hipGetLastError(); return GRIM_ERR_ALLOC; }
    if (hipMemcpy(ptr, words.data(), words.size() * 4, hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipFree(ptr);
        return GRIM_ERR_DEVICE;
    }
    P->d_words = static_cast<uint32_t *>(ptr);
    *out = P.release();
    return GRIM_OK;
}

void grim_bcr_conv_plan_free(grim_bcr_conv_plan *P) {
    if (!P) return;
    if (P->d_words) (void)hipFree(P->d_words);
    delete P;
}

grim_status grim_bcr_conv2d_plan(const grim_bcr_conv_plan *P, const void *F_dev, int32_t batch, int64_t f_image_stride,
                                 const float *bias_dev, int32_t relu, void *out_dev, grim_dtype out_dt, int64_t ldo,
                                 int64_t out_image_stride, void *hip_stream) {
    if (!P || !F_dev || !out_dev) return GRIM_ERR_NULL;
    const int64_t Ho = (P->H + P->stride - 1) / P->stride, Wo = (P->W + P->stride - 1) / P->stride;
    const int64_t M = P->A->M;
    if (batch < 1 || ldo < Ho * Wo) return GRIM_ERR_SHAPE;
    if (batch > 1 && (f_image_stride < (int64_t)P->Cin * P->H * P->W || out_image_stride < (M - 1) * ldo + Ho * Wo))
        return GRIM_ERR_SHAPE;
    if (out_dt != GRIM_F32 && out_dt != GRIM_F16 && out_dt != GRIM_BF16) return GRIM_ERR_DTYPE;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != P->device) { (void)hipGetLastError(); return GRIM_ERR_DEVICE; }
    if (P->stride == 1) {
        const grim_status st = launch_conv_wide(P->A, F_dev, P->Cin, P->H, P->W, P->kh, P->kw, batch, f_image_stride, bias_dev,
                                                relu ? 1 : 0, out_dev, (int32_t)out_dt, ldo, out_image_stride,
                                                static_cast<hipStream_t>(hip_stream));
        if (st != GRIM_ERR_UNSUPPORTED) return st;
    }
    return launch_conv_gather(P->A, F_dev, P->Cin, P->H, P->W, P->kh, P->kw, bias_dev, relu ? 1 : 0, out_dev, (int32_t)out_dt,
                              ldo, static_cast<hipStream_t>(hip_stream), batch, P->stride, f_image_stride, out_image_stride,
                              P->d_words);
}

const char *grim_bcr_conv2d_kernel_name(const grim_bcr_matrix *A, int32_t Cin, int32_t H, int32_t W, int32_t kh, int32_t kw,
                                        int32_t batch, int32_t stride) {
    if (!A || !A->on_device || Cin < 1 || H < 1 || W < 1 || kh < 1 || kw < 1 || batch < 1 || (int64_t)Cin * kh * kw != A->K)
        return "none";
    // operands as tests and benchmarks pass them: 16-byte aligned, dense images one after the other
    const int64_t HW = (int64_t)H * W;
    void *aligned = reinterpret_cast<void *>(uintptr_t(256));
    if (stride == 1 && conv_wide_applies(A, aligned, Cin, H, W, kh, kw, batch, Cin * HW, aligned, GRIM_F32, HW, A->M * HW))
        return "bcr_conv_wide";
    return A->gather.present ? "bcr_conv_gather" : "none";
}

grim_status grim_lstm_cell(const float *gates_dev, int64_t ldg, const float *bias_dev, float *c_dev, int64_t ldc,
                           void *h_dev, grim_dtype dt, int64_t ldh, float *h32_dev, int64_t ldh32, int64_t H,
                           int32_t batch, void *hip_stream) {
    if (!gates_dev || !c_dev) return GRIM_ERR_NULL;
    if (H < 1 || batch < 1 || ldg < batch || ldc < batch || (h_dev && ldh < batch) || (h32_dev && ldh32 < batch))
        return GRIM_ERR_SHAPE;
    if (H > (int64_t(1) << 40) / batch) return GRIM_ERR_SHAPE;
    if (dt != GRIM_F32 && dt != GRIM_F16 && dt != GRIM_BF16) return GRIM_ERR_DTYPE;
    return launch_lstm_cell(gates_dev, ldg, bias_dev, c_dev, ldc, h_dev, dt, ldh, h32_dev, ldh32, H, batch,
                            static_cast<hipStream_t>(hip_stream));
}

grim_status grim_bcr_lstm_step(const grim_bcr_matrix *A, const void *xh_dev, int32_t batch, int64_t ldx,
                               float *gates_dev, int64_t ldg, const float *bias_dev, float *c_dev, int64_t ldc,
                               void *h_dev, int64_t ldh, float *h32_dev, int64_t ldh32, void *hip_stream) {
    if (!A || !xh_dev || !gates_dev || !c_dev) return GRIM_ERR_NULL;
    if (A->M % 4 != 0) return GRIM_ERR_SHAPE;
    const int64_t H = A->M / 4;
    if (batch < 1 || ldc < batch || (h_dev && ldh < batch) || (h32_dev && ldh32 < batch)) return GRIM_ERR_SHAPE;
    if (A->gemv.present && spmv_cell_batch_ok(H, A->BR, batch)) {
        // One launch: the cell in the epilogue of the gate product, a set of workgroups per column of xh.  Workgroups
        // then write h while others may still read the input vectors, so the new h must not land in what this step reads.
        grim_status st0 = check_call(A, xh_dev, batch, ldx, gates_dev, ldg);
        if (st0 != GRIM_OK) return st0;
        const int esz = dtype_size(A->dtype);
        const bool aliased = h_dev && ranges_overlap(xh_dev, ((A->K - 1) * ldx + batch) * esz, h_dev, ((H - 1) * ldh + batch) * esz);
        if (!aliased) {
            // (a matrix stored in its original strip order spares the step kernel the look-up its weight fetch waits for)
            RnnCell cell{A->order_identity ? nullptr : A->dev.strip_pos, nullptr, bias_dev, nullptr, c_dev, h_dev, h32_dev, ldc, ldh, ldh32,
                         (int32_t)H, A->dtype};
            st0 = launch_spmv_cell(1, desc_of(A), nullptr, A->M, A->K, A->BR, A->BC, A->dtype, A->gemv.uniform_kr,
                                   A->gemv.uniform_kc, xh_dev, 0, batch, ldx, gates_dev, 0, ldg, cell, static_cast<hipStream_t>(hip_stream));
            if (st0 != GRIM_ERR_UNSUPPORTED) return st0;
        }
    }
    grim_status st = batch <= 8 ? grim_bcr_spmv(A, xh_dev, batch, ldx, gates_dev, ldg, hip_stream)
                                : grim_bcr_spmm(A, xh_dev, batch, ldx, gates_dev, ldg, hip_stream);
    if (st != GRIM_OK) return st;
    return grim_lstm_cell(gates_dev, ldg, bias_dev, c_dev, ldc, h_dev, (grim_dtype)A->dtype, ldh, h32_dev, ldh32, H, batch,
                          hip_stream);
}

int32_t grim_bcr_rnn_step_launches(const grim_bcr_matrix *A, const grim_bcr_matrix *Ah, int32_t batch) {
    if (!A || batch < 1 || !A->on_device) return 0;
    if (!Ah) {
        if (A->M % 4 != 0) return 0;
        const bool fused = A->gemv.present && spmv_cell_batch_ok(A->M / 4, A->BR, batch) &&
                           spmv_cell_applies(1, A->M, A->K, A->BR, A->BC, A->dtype, A->gemv.uniform_kr, A->gemv.uniform_kc, A->M / 4);
        return fused ? 1 : 2;
    }
    if (A->M != Ah->M || A->M % 3 != 0 || Ah->K != A->M / 3 || A->dtype != Ah->dtype || !Ah->on_device) return 0;
    const bool same = A->K == Ah->K && A->BR == Ah->BR && A->BC == Ah->BC && A->gemv.present && Ah->gemv.present;
    const bool fused = spmv_cell_batch_ok(A->M / 3, A->BR, batch) && same && A->gemv.uniform_kr == Ah->gemv.uniform_kr && A->gemv.uniform_kc == Ah->gemv.uniform_kc &&
                       spmv_cell_applies(2, A->M, A->K, A->BR, A->BC, A->dtype, A->gemv.uniform_kr, A->gemv.uniform_kc, A->M / 3);
    if (fused) return 1;
    // both products in one launch (SpMV kernels up to 8 columns when the matrices have one shape; the row-gathering
    // kernel for 4 .. 60 columns in multiples of 4), then the cell; otherwise a launch per product
    const bool one_spmv = batch <= 8 && same && A->K * batch * dtype_size(A->dtype) <= kGemvMaxXBytes;
    const bool one_gather = batch < 64 && batch % 4 == 0 && A->gather.present && Ah->gather.present &&
                            A->gather.nstrips == Ah->gather.nstrips;
    return one_spmv || one_gather ? 2 : 3;
}

// exchange words of the sequence kernel: allocated with the first sequence call on a matrix, freed with the matrix
static grim_status seq_exchange_of(const grim_bcr_matrix *A, int64_t H, void **out) {
    std::lock_guard<std::mutex> hold(A->seq_lock);
    if (!A->seq_exch) {
        void *ptr = nullptr;
        // two slots of at most one word per hidden unit and sequence, for the largest batch
        if (hipMalloc(&ptr, (size_t)(2 * H) * kSeqMaxBatch * 8) != hipSuccess) {
            (void)hipGetLastError();
            return GRIM_ERR_ALLOC;
        }
        A->seq_exch = ptr;
    }
    *out = A->seq_exch;
    return GRIM_OK;
}

static grim_status seq_check(const grim_bcr_matrix *A, const void *xs, int32_t T, int32_t batch, const void *h0,
                             const float *state, const void *hs, const int32_t *status) {
    if (!A || !xs || !h0 || !state || !hs || !status) return GRIM_ERR_NULL;
    if (T < 1 || batch < 1) return GRIM_ERR_SHAPE;
    if (!A->on_device) return GRIM_ERR_DEVICE;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != A->device) return GRIM_ERR_DEVICE;
    return GRIM_OK;
}

int32_t grim_bcr_rnn_sequence_supported(const grim_bcr_matrix *A, const grim_bcr_matrix *Ah) {
    return grim_bcr_rnn_sequence_batch_supported(A, Ah, 1);
}

int32_t grim_bcr_rnn_sequence_batch_supported(const grim_bcr_matrix *A, const grim_bcr_matrix *Ah, int32_t batch) {
    if (!A || !A->on_device || !A->gemv.present) return 0;
    if (!Ah) {
        if (A->M % 4 != 0 || A->K <= A->M / 4) return 0;
        const int64_t H = A->M / 4;
        return rnn_seq_applies(1, A->BR, A->BC, A->dtype, A->gemv.uniform_kr, A->gemv.uniform_kc, A->K, 0, A->K - H, H, batch) ? 1 : 0;
    }
    if (!Ah->on_device || !Ah->gemv.present || A->M != Ah->M || A->M % 3 != 0 || Ah->K != A->M / 3) return 0;
    if (A->dtype != Ah->dtype || A->BR != Ah->BR || A->BC != Ah->BC || A->gemv.uniform_kr != Ah->gemv.uniform_kr ||
        A->gemv.uniform_kc != Ah->gemv.uniform_kc)
        return 0;
    return rnn_seq_applies(2, A->BR, A->BC, A->dtype, A->gemv.uniform_kr, A->gemv.uniform_kc, A->K, Ah->K, A->K, Ah->K, batch) ? 1 : 0;
}

grim_status grim_bcr_lstm_sequence(const grim_bcr_matrix *A, const void *xs_dev, int64_t ldxs, int32_t T,
                                   const float *bias_dev, const void *h0_dev, float *c_dev, void *hs_dev, int64_t ldhs,
                                   float *hs32_dev, int64_t ldhs32, int32_t *status_dev, uint32_t max_polls,
                                   void *hip_stream) {
    return grim_bcr_lstm_sequence_batch(A, xs_dev, ldxs, T, 1, bias_dev, h0_dev, c_dev, hs_dev, ldhs, hs32_dev, ldhs32,
                                        status_dev, max_polls, hip_stream);
}

grim_status grim_bcr_lstm_sequence_batch(const grim_bcr_matrix *A, const void *xs_dev, int64_t ldxs, int32_t T, int32_t batch,
                                         const float *bias_dev, const void *h0_dev, float *c_dev, void *hs_dev, int64_t ldhs,
                                         float *hs32_dev, int64_t ldhs32, int32_t *status_dev, uint32_t max_polls,
                                         void *hip_stream) {
    grim_status st = seq_check(A, xs_dev, T, batch, h0_dev, c_dev, hs_dev, status_dev);
    if (st != GRIM_OK) return st;
    if (A->M % 4 != 0 || A->K <= A->M / 4) return GRIM_ERR_SHAPE;
    const int64_t H = A->M / 4, I = A->K - H;
    if (ldxs < I || ldhs < H || (hs32_dev && ldhs32 < H)) return GRIM_ERR_SHAPE;
    if (!grim_bcr_rnn_sequence_batch_supported(A, nullptr, batch)) return GRIM_ERR_UNSUPPORTED;
    void *exch = nullptr;
    st = seq_exchange_of(A, H, &exch);
    if (st != GRIM_OK) return st;
    return launch_rnn_seq(1, desc_of(A), nullptr, A->dev.strip_pos, nullptr, A->BR, A->BC, A->dtype, A->gemv.uniform_kr,
                          A->gemv.uniform_kc, A->K, 0, I, H, T, batch, xs_dev, ldxs, h0_dev, bias_dev, nullptr, c_dev, hs_dev,
                          ldhs, hs32_dev, ldhs32, exch, status_dev, max_polls, static_cast<hipStream_t>(hip_stream));
}

grim_status grim_bcr_lstm_sequence_noalloc(const grim_bcr_matrix *A, const void *xs_dev, int64_t ldxs, int32_t T,
                                           const float *bias_dev, const void *h0_dev, float *c_dev, void *hs_dev,
                                           int64_t ldhs, float *hs32_dev, int64_t ldhs32, int32_t *status_dev,
                                           uint32_t max_polls, void *hip_stream) {
    grim_status st = seq_check(A, xs_dev, T, 1, h0_dev, c_dev, hs_dev, status_dev);
    if (st != GRIM_OK) return st;
    if (A->M % 4 != 0 || A->K <= A->M / 4) return GRIM_ERR_SHAPE;
    const int64_t H = A->M / 4, I = A->K - H;
    if (ldxs < I || ldhs < H || (hs32_dev && ldhs32 < H)) return GRIM_ERR_SHAPE;
    if (H > kSeqMaxH) return GRIM_ERR_UNSUPPORTED;                 // beyond the static exchange words
    if (!grim_bcr_rnn_sequence_supported(A, nullptr)) return GRIM_ERR_UNSUPPORTED;
    void *exch = nullptr;
    st = rnn_seq_static_exchange(&exch);
    if (st != GRIM_OK) return st;
    return launch_rnn_seq(1, desc_of(A), nullptr, A->dev.strip_pos, nullptr, A->BR, A->BC, A->dtype, A->gemv.uniform_kr,
                          A->gemv.uniform_kc, A->K, 0, I, H, T, 1, xs_dev, ldxs, h0_dev, bias_dev, nullptr, c_dev, hs_dev, ldhs,
                          hs32_dev, ldhs32, exch, status_dev, max_polls, static_cast<hipStream_t>(hip_stream));
}

grim_status grim_bcr_gru_sequence(const grim_bcr_matrix *Ai, const grim_bcr_matrix *Ah, const void *xs_dev, int64_t ldxs,
                                  int32_t T, const float *bias_i_dev, const float *bias_h_dev, const void *h0_dev,
                                  float *h32_dev, void *hs_dev, int64_t ldhs, float *hs32_dev, int64_t ldhs32,
                                  int32_t *status_dev, uint32_t max_polls, void *hip_stream) {
    return grim_bcr_gru_sequence_batch(Ai, Ah, xs_dev, ldxs, T, 1, bias_i_dev, bias_h_dev, h0_dev, h32_dev, hs_dev, ldhs,
                                       hs32_dev, ldhs32, status_dev, max_polls, hip_stream);
}

grim_status grim_bcr_gru_sequence_batch(const grim_bcr_matrix *Ai, const grim_bcr_matrix *Ah, const void *xs_dev, int64_t ldxs,
                                        int32_t T, int32_t batch, const float *bias_i_dev, const float *bias_h_dev,
                                        const void *h0_dev, float *h32_dev, void *hs_dev, int64_t ldhs, float *hs32_dev,
                                        int64_t ldhs32, int32_t *status_dev, uint32_t max_polls, void *hip_stream) {
    grim_status st = seq_check(Ai, xs_dev, T, batch, h0_dev, h32_dev, hs_dev, status_dev);
    if (st != GRIM_OK) return st;
    if (!Ah) return GRIM_ERR_NULL;
    if (Ai->M != Ah->M || Ai->M % 3 != 0 || Ah->K != Ai->M / 3) return GRIM_ERR_SHAPE;
    if (Ai->dtype != Ah->dtype) return GRIM_ERR_DTYPE;
    if (!Ah->on_device || Ah->device != Ai->device) return GRIM_ERR_DEVICE;
    const int64_t H = Ah->K, I = Ai->K;
    if (ldxs < I || ldhs < H || (hs32_dev && ldhs32 < H)) return GRIM_ERR_SHAPE;
    if (!grim_bcr_rnn_sequence_batch_supported(Ai, Ah, batch)) return GRIM_ERR_UNSUPPORTED;
    void *exch = nullptr;
    st = seq_exchange_of(Ah, H, &exch);
    if (st != GRIM_OK) return st;
    const GemvDesc dh = desc_of(Ah);
    return launch_rnn_seq(2, desc_of(Ai), &dh, Ai->dev.strip_pos, Ah->dev.strip_pos, Ai->BR, Ai->BC, Ai->dtype,
                          Ai->gemv.uniform_kr, Ai->gemv.uniform_kc, I, H, I, H, T, batch, xs_dev, ldxs, h0_dev, bias_i_dev, bias_h_dev,
                          h32_dev, hs_dev, ldhs, hs32_dev, ldhs32, exch, status_dev, max_polls,
                          static_cast<hipStream_t>(hip_stream));
}

grim_status grim_gru_cell(const float *gi_dev, int64_t ldgi, const float *gh_dev, int64_t ldgh, const float *bias_i_dev,
                          const float *bias_h_dev, float *h32_dev, int64_t ldh32, void *h_dev, grim_dtype dt, int64_t ldh,
                          int64_t H, int32_t batch, void *hip_stream) {
    if (!gi_dev || !gh_dev || !h32_dev) return GRIM_ERR_NULL;
    if (H < 1 || batch < 1 || ldgi < batch || ldgh < batch || ldh32 < batch || (h_dev && ldh < batch)) return GRIM_ERR_SHAPE;
    if (H > (int64_t(1) << 40) / batch) return GRIM_ERR_SHAPE;
    if (dt != GRIM_F32 && dt != GRIM_F16 && dt != GRIM_BF16) return GRIM_ERR_DTYPE;
    return launch_gru_cell(gi_dev, ldgi, gh_dev, ldgh, bias_i_dev, bias_h_dev, h32_dev, ldh32, h_dev, dt, ldh, H, batch,
                           static_cast<hipStream_t>(hip_stream));
}

grim_status grim_bcr_gru_step(const grim_bcr_matrix *Ai, const grim_bcr_matrix *Ah, const void *x_dev, int64_t ldx,
                              const void *hin_dev, int64_t ldhin, int32_t batch, float *gi_dev, int64_t ldgi,
                              float *gh_dev, int64_t ldgh, const float *bias_i_dev, const float *bias_h_dev,
                              float *h32_dev, int64_t ldh32, void *hout_dev, int64_t ldhout, void *hip_stream) {
    if (!Ai || !Ah || !x_dev || !hin_dev || !gi_dev || !gh_dev || !h32_dev) return GRIM_ERR_NULL;
    if (Ai->M != Ah->M || Ai->M % 3 != 0 || Ah->K != Ai->M / 3) return GRIM_ERR_SHAPE;
    if (Ai->dtype != Ah->dtype) return GRIM_ERR_DTYPE;
    const int64_t H = Ai->M / 3;
    if (batch < 1 || ldh32 < batch || (hout_dev && ldhout < batch)) return GRIM_ERR_SHAPE;
    grim_status st = check_call(Ai, x_dev, batch, ldx, gi_dev, ldgi);
    if (st == GRIM_OK) st = check_call(Ah, hin_dev, batch, ldhin, gh_dev, ldgh);
    if (st != GRIM_OK) return st;
    // Both products in one launch when the two matrices have one shape and the SpMV kernels take
    // them: the second operand / result is addressed as the first plus a stride (of either sign).
    const int esz = dtype_size(Ai->dtype);
    const ptrdiff_t xd = static_cast<const char *>(hin_dev) - static_cast<const char *>(x_dev);
    const ptrdiff_t yd = reinterpret_cast<const char *>(gh_dev) - reinterpret_cast<const char *>(gi_dev);
    // (8 columns in 16-byte-aligned rows are quicker on the matrix cores, as for a lone product)
    if (spmv_cell_batch_ok(H, Ai->BR, batch) && Ai->K == Ah->K && Ai->BR == Ah->BR && Ai->BC == Ah->BC && Ai->gemv.present && Ah->gemv.present &&
        Ai->gemv.uniform_kr == Ah->gemv.uniform_kr && Ai->gemv.uniform_kc == Ah->gemv.uniform_kc && ldx == ldhin && ldgi == ldgh &&
        xd % esz == 0 && yd % 4 == 0) {
        // One launch: both gate products with the cell in the epilogue.  The new state must not land in the vector
        // the hidden-side product reads (workgroups write it while others may still read).
        const bool aliased = hout_dev && (ranges_overlap(hin_dev, ((Ah->K - 1) * ldhin + batch) * esz, hout_dev, ((H - 1) * ldhout + batch) * esz) ||
                                          ranges_overlap(x_dev, ((Ai->K - 1) * ldx + batch) * esz, hout_dev, ((H - 1) * ldhout + batch) * esz));
        if (!aliased) {
            const GemvDesc di = desc_of(Ai), dh = desc_of(Ah);
            RnnCell cell{Ai->order_identity ? nullptr : Ai->dev.strip_pos, Ah->order_identity ? nullptr : Ah->dev.strip_pos, bias_i_dev, bias_h_dev, h32_dev, hout_dev, nullptr, ldh32, ldhout, 0,
                         (int32_t)H, Ai->dtype};
            st = launch_spmv_cell(2, di, &dh, Ai->M, Ai->K, Ai->BR, Ai->BC, Ai->dtype, Ai->gemv.uniform_kr, Ai->gemv.uniform_kc,
                                  x_dev, xd / esz, batch, ldx, gi_dev, yd / 4, ldgi, cell, static_cast<hipStream_t>(hip_stream));
            if (st != GRIM_ERR_UNSUPPORTED) return st;
        }
    }
    const bool eight_on_matrix_cores = ldx == ldhin && ldgi == ldgh && skinny_on_matrix_cores(Ai, x_dev, batch, ldx, 2) &&
                                       skinny_on_matrix_cores(Ah, hin_dev, batch, ldx, 2) &&
                                       gather_pair_applies(Ai, x_dev, Ah, hin_dev, batch, ldx);
    if (!eight_on_matrix_cores && batch <= 8 && Ai->K == Ah->K && Ai->BR == Ah->BR && Ai->BC == Ah->BC && gemv_ok(Ai, batch) &&
        gemv_ok(Ah, batch) && ldx == ldhin && ldgi == ldgh && xd % esz == 0 && yd % 4 == 0) {
        const GemvDesc di = desc_of(Ai), dh = desc_of(Ah);
        const bool same = Ai->gemv.uniform_kr == Ah->gemv.uniform_kr && Ai->gemv.uniform_kc == Ah->gemv.uniform_kc;
        st = launch_spmv(nullptr, di, &dh, 2, Ai->M, Ai->K, Ai->BR, Ai->BC, Ai->dtype, same ? Ai->gemv.uniform_kr : -1,
                         same ? Ai->gemv.uniform_kc : -1, std::min(Ai->gemv.vec, Ah->gemv.vec),
                         std::max(Ai->gemv.krmax, Ah->gemv.krmax), std::max(Ai->gemv.kcmax, Ah->gemv.kcmax), x_dev, xd / esz,
                         batch, ldx, gi_dev, yd / 4, ldgi, static_cast<hipStream_t>(hip_stream));
    } else if (ldx == ldhin && ldgi == ldgh && gather_pair_applies(Ai, x_dev, Ah, hin_dev, batch, ldx)) {
        // 4 .. 60 columns on the matrix cores: one launch of the row-gathering kernel, grid.y = product
        st = launch_spmm_gather(Ai, x_dev, batch, ldx, gi_dev, ldgi, static_cast<hipStream_t>(hip_stream), Ah, hin_dev, gh_dev);
    } else {
        st = grim_bcr_spmm(Ai, x_dev, batch, ldx, gi_dev, ldgi, hip_stream);
        if (st == GRIM_OK) st = grim_bcr_spmm(Ah, hin_dev, batch, ldhin, gh_dev, ldgh, hip_stream);
    }
    if (st != GRIM_OK) return st;
    return grim_gru_cell(gi_dev, ldgi, gh_dev, ldgh, bias_i_dev, bias_h_dev, h32_dev, ldh32, hout_dev, (grim_dtype)Ai->dtype,
                         ldhout, H, batch, hip_stream);
}

grim_status grim_bcr_group_create(const grim_bcr_matrix *const *mats, int32_t count, grim_bcr_group **out) {
    if (out) *out = nullptr;
    if (!mats || !out) return GRIM_ERR_NULL;
    if (count < 1 || count > 65535) return GRIM_ERR_SHAPE;   // grid.y = matrix
    for (int32_t i = 0; i < count; ++i)
        if (!mats[i]) return GRIM_ERR_NULL;
    const grim_bcr_matrix *A0 = mats[0];
    int dev = -1;
    if (!A0->on_device || hipGetDevice(&dev) != hipSuccess || dev != A0->device) return GRIM_ERR_DEVICE;
    if (!A0->gemv.present) return GRIM_ERR_UNSUPPORTED;
    grim_bcr_group *G = nullptr;
    std::vector<GemvDesc> table;
    try {
        G = new grim_bcr_group();
        table.resize(count);
    } catch (const std::bad_alloc &) {
        delete G;
        return GRIM_ERR_ALLOC;
    }
    G->count = count; G->M = A0->M; G->K = A0->K; G->BR = A0->BR; G->BC = A0->BC; G->dtype = A0->dtype;
    G->nbr = A0->nbr; G->nbc = A0->nbc; G->device = dev;
    G->uniform_kr = A0->gemv.uniform_kr; G->uniform_kc = A0->gemv.uniform_kc; G->vec = A0->gemv.vec;
    G->krmax = A0->gemv.krmax; G->kcmax = A0->gemv.kcmax;
    for (int32_t i = 0; i < count; ++i) {
        const grim_bcr_matrix *A = mats[i];
        if (A->M != G->M || A->K != G->K || A->BR != G->BR || A->BC != G->BC || A->dtype != G->dtype) { delete G; return GRIM_ERR_SHAPE; }
        if (!A->on_device || A->device != dev) { delete G; return GRIM_ERR_DEVICE; }
        if (!A->gemv.present) { delete G; return GRIM_ERR_UNSUPPORTED; }
        if (A->gemv.uniform_kr != G->uniform_kr || A->gemv.uniform_kc != G->uniform_kc) G->uniform_kr = G->uniform_kc = -1;
        G->vec = std::min(G->vec, A->gemv.vec);
        G->krmax = std::max(G->krmax, A->gemv.krmax);
        G->kcmax = std::max(G->kcmax, A->gemv.kcmax);
        table[i] = desc_of(A);
    }
    if (hipMalloc(reinterpret_cast<void **>(&G->d_table), sizeof(GemvDesc) * count) != hipSuccess) { (void)hipGetLastError(); delete G; return GRIM_ERR_ALLOC; }
    if (hipMemcpy(G->d_table, table.data(), sizeof(GemvDesc) * count, hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipGetLastError(); (void)hipFree(G->d_table); delete G; return GRIM_ERR_DEVICE;
    }
    *out = G;
    return GRIM_OK;
}

grim_status grim_bcr_spmv_batched(const grim_bcr_group *G, const void *x_dev, int64_t x_stride, int32_t batch, int64_t ldx,
                                  float *y_dev, int64_t y_stride, int64_t ldy, void *hip_stream) {
    if (!G || !x_dev || !y_dev) return GRIM_ERR_NULL;
    if (batch < 1 || batch > 8 || ldx < batch || ldy < batch || x_stride < 0 || y_stride < 0) return GRIM_ERR_SHAPE;
    if (G->K * batch * dtype_size(G->dtype) > kGemvMaxXBytes) return GRIM_ERR_UNSUPPORTED;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != G->device) return GRIM_ERR_DEVICE;
    GemvDesc none{nullptr, nullptr, nullptr, nullptr};
    return launch_spmv(G->d_table, none, nullptr, G->count, G->M, G->K, G->BR, G->BC, G->dtype, G->uniform_kr, G->uniform_kc, G->vec, G->krmax, G->kcmax,
                       x_dev, x_stride, batch, ldx, y_dev, y_stride, ldy, static_cast<hipStream_t>(hip_stream));
}

void grim_bcr_group_free(grim_bcr_group *G) {
    if (!G) return;
    if (G->d_table) (void)hipFree(G->d_table);
    delete G;
}

void grim_bcr_free(grim_bcr_matrix *A) {
    if (!A) return;
    if (A->seq_exch) (void)hipFree(A->seq_exch);
    if (A->on_device && A->dev.strip_order) (void)hipFree(A->dev.strip_order);   // base of the slab
    delete A;
}

const char *grim_status_str(grim_status s) {
    switch (s) {
        case GRIM_OK: return "GRIM_OK";
        case GRIM_ERR_NULL: return "GRIM_ERR_NULL: required pointer is NULL";
        case GRIM_ERR_SHAPE: return "GRIM_ERR_SHAPE: invalid shape, block size, leading dimension or batch";
        case GRIM_ERR_INDEX: return "GRIM_ERR_INDEX: malformed kept-row / kept-column index sets";
        case GRIM_ERR_DTYPE: return "GRIM_ERR_DTYPE: unknown element type";
        case GRIM_ERR_ALLOC: return "GRIM_ERR_ALLOC: allocation failed";
        case GRIM_ERR_DEVICE: return "GRIM_ERR_DEVICE: HIP failure, no GPU, wrong current device, or host-only matrix";
        case GRIM_ERR_UNSUPPORTED: return "GRIM_ERR_UNSUPPORTED: no kernel covers this request";
    }
    return "unknown grim_status";
}

}  // extern "C"

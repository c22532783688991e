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
#include "spmm_wide_kernel.hpp"
#include "spmm_gather_kernel.hpp"

namespace grim {

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

// The wide-tile workgroups and, behind them in the same launch, the row-gathering workgroups of the columns they leave
// over (eight-wave form, 16-byte-aligned rows).  A launch of its own for those few columns costs a dispatch and runs
// its short chains of dependent fetches on an otherwise idle GPU; here they start on whichever compute unit finishes
// its wide workgroup first, while the others are still busy.  All twelve waves of a workgroup split the strip's steps
// (the kernel of its own uses eight): at 40-odd steps per strip a wave then has one batch of loads, not two.
template <bool BF16, int BR, int NT>
__global__ void __launch_bounds__(kWideThreads) bcr_spmm_wide_rest(WideParams wp, GatherParams gp, int wide_wgs) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    if ((int)blockIdx.x < wide_wgs) {
        wide_body<BF16, BR, NT, false>(wp, lds, blockIdx.x);
        return;
    }
    // (a workgroup number past the last (tile, strip) leaves as a whole: no wave may wait at a barrier others skip)
    const int vblock = (int)blockIdx.x - wide_wgs;
    int tile, unit;
    if (!xcd_map_at(gp.map, vblock, gp.ntiles, &tile, &unit) || unit >= gp.nbr) return;
    gather_body<BF16, true, false, false, true, kWideMulWaves + kWideFetchWaves>(gp, lds, vblock, 0);
}

template <bool BF16, int BR, int NT>
static grim_status launch_wide_rest_inst(const WideParams &wp, const GatherParams &gp, size_t lds, int64_t wide_wgs, int64_t rest_wgs,
                                         hipStream_t stream) {
    auto kern = bcr_spmm_wide_rest<BF16, BR, NT>;
    static std::atomic<bool> attr_done{false};
    if (lds > 64 * 1024 && !attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) {
            (void)hipGetLastError();
            return GRIM_ERR_DEVICE;
        }
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(wide_wgs + rest_wgs)), dim3(kWideThreads), lds, stream, wp, gp, (int)wide_wgs);
    return hipGetLastError() == hipSuccess ? GRIM_OK : GRIM_ERR_DEVICE;
}

static grim_status wide_setup(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, float *Y, int64_t ldy, int32_t tile_n,
                              WideParams *out, int *tn_out, int64_t *nwg_out);

grim_status launch_spmm_wide(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, float *Y, int64_t ldy,
                             int32_t tile_n, hipStream_t stream) {
    WideParams p;
    int tn = 0;
    int64_t nwg = 0;
    const grim_status st = wide_setup(A, X, N, ldx, Y, ldy, tile_n, &p, &tn, &nwg);
    if (st != GRIM_OK) return st;
    const size_t lds = (size_t)wide_lds_bytes(A, tn);
    const bool bf = A->dtype == GRIM_BF16;
    if (A->BR == 16) {
        if (tn == 128) return bf ? launch_wide_inst<true, 16, 8>(p, lds, nwg, stream) : launch_wide_inst<false, 16, 8>(p, lds, nwg, stream);
        return bf ? launch_wide_inst<true, 16, 12>(p, lds, nwg, stream) : launch_wide_inst<false, 16, 12>(p, lds, nwg, stream);
    }
    return bf ? launch_wide_inst<true, 32, 3>(p, lds, nwg, stream) : launch_wide_inst<false, 32, 3>(p, lds, nwg, stream);
}

// Columns [0, wide_cols) on the wide-tile workgroups and [wide_cols, N) on row-gathering workgroups, one launch.
// GRIM_ERR_UNSUPPORTED (nothing enqueued) when the rest does not take the kernel form this launch is built for.
grim_status launch_spmm_wide_with_rest(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, float *Y, int64_t ldy,
                                       int32_t tile_n, int64_t wide_cols, hipStream_t stream) {
    if (wide_cols <= 0 || wide_cols >= N) return GRIM_ERR_UNSUPPORTED;
    WideParams wp;
    int tn = 0;
    int64_t wide_wgs = 0;
    grim_status st = wide_setup(A, X, wide_cols, ldx, Y, ldy, tile_n, &wp, &tn, &wide_wgs);
    if (st != GRIM_OK) return st;
    GatherParams gp;
    GatherForm form;
    const char *x_rest = static_cast<const char *>(X) + wide_cols * dtype_size(A->dtype);
    st = gather_setup(A, x_rest, N - wide_cols, ldx, Y + wide_cols, ldy, nullptr, nullptr, nullptr, &gp, &form);
    if (st != GRIM_OK) return st;
    if (!form.wide || form.narrow || form.solo || !form.eight) return GRIM_ERR_UNSUPPORTED;
    if (wide_wgs + form.nwg > 0x7fffffff) return GRIM_ERR_SHAPE;
    const size_t lds = std::max<size_t>((size_t)wide_lds_bytes(A, tn), (size_t)(kWideMulWaves + kWideFetchWaves) * 8192);
    const bool bf = A->dtype == GRIM_BF16;
    if (A->BR == 16) {
        if (tn == 128)
            return bf ? launch_wide_rest_inst<true, 16, 8>(wp, gp, lds, wide_wgs, form.nwg, stream)
                      : launch_wide_rest_inst<false, 16, 8>(wp, gp, lds, wide_wgs, form.nwg, stream);
        return bf ? launch_wide_rest_inst<true, 16, 12>(wp, gp, lds, wide_wgs, form.nwg, stream)
                  : launch_wide_rest_inst<false, 16, 12>(wp, gp, lds, wide_wgs, form.nwg, stream);
    }
    return bf ? launch_wide_rest_inst<true, 32, 3>(wp, gp, lds, wide_wgs, form.nwg, stream)
              : launch_wide_rest_inst<false, 32, 3>(wp, gp, lds, wide_wgs, form.nwg, stream);
}

static grim_status wide_setup(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, float *Y, int64_t ldy, int32_t tile_n,
                              WideParams *out, int *tn_out, int64_t *nwg_out) {
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
    *out = p;
    *tn_out = tn;
    *nwg_out = nwg;
    return GRIM_OK;
}

}  // namespace grim

#include "spmm_gather_kernel.hpp"

namespace grim {

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

// Parameters, grid and kernel form of a launch (see launch_spmm_gather); GRIM_ERR_UNSUPPORTED when the kernel does not apply.
grim_status gather_setup(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, float *Y, int64_t ldy,
                         const grim_bcr_matrix *A2, const void *X2, float *Y2, GatherParams *out, GatherForm *form) {
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
    form->narrow = narrow;
    form->solo = solo;
    form->eight = eight;
    form->wide = N % 8 == 0 && ldx % 8 == 0 && reinterpret_cast<uintptr_t>(X) % 16 == 0 &&
                 (!A2 || reinterpret_cast<uintptr_t>(X2) % 16 == 0);
    form->nwg = nwg;
    *out = p;
    return GRIM_OK;
}

grim_status launch_spmm_gather(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, float *Y, int64_t ldy,
                               hipStream_t stream, const grim_bcr_matrix *A2, const void *X2, float *Y2) {
    GatherParams p;
    GatherForm form;
    const grim_status st = gather_setup(A, X, N, ldx, Y, ldy, A2, X2, Y2, &p, &form);
    if (st != GRIM_OK) return st;
    const bool narrow = form.narrow, solo = form.solo, eight = form.eight, wide = form.wide;
    const int64_t nwg = form.nwg;
    const size_t lds = (eight ? kGatherLongWaves : 4) * 8192;
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

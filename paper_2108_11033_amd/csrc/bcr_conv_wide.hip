// Convolution on the wide-tile staged kernel, the im2col matrix never formed (Section 3.1: CONV = filter matrix x
// im2col matrix; Section 4.5: that matrix need not exist in memory).  For layers with many output positions
// (large maps, batches): a workgroup owns a tile of 96-192 consecutive positions of the batch and 16 row strips; its
// fetching waves build the K rows of the tile -- row k is channel k / (kh kw) of the feature map shifted by tap
// k % (kh kw), zero outside the image -- in LDS with one 16-byte load per 8 positions, and the multiplying waves
// run exactly as for a matrix X in memory.  Every pixel is fetched kh * kw times, but from the caches: HBM sees the
// feature maps once instead of a matrix kh * kw times their size.
// Launches: whole rounds of 256 workgroups at the widest tile; the remaining positions go to the row-gathering
// convolution on a position range, or to 32-column tiles of this kernel when that does not apply (a partial round of
// wide tiles would cost as much as a full one).  Small layers stay on the row-gathering convolution kernel.
#include <algorithm>
#include <atomic>

#include "spmm_wide_kernel.hpp"
#include "conv_gather_kernel.hpp"

namespace grim {

// tile widths compiled for the convolution: the widest for the whole rounds, 32 columns for what is left
constexpr int kConvWideRestTile = 32;

static size_t conv_wide_lds(const grim_bcr_matrix *A, int tn, int KK) {
    // two stages, the (tap, piece) mask table, four per-chunk row tables
    return 2 * (size_t)wide_stage_bytes(A->mmaw.chunk_rows, tn, A->mmaw.amax[2]) + (size_t)(KK + 1) * (tn / 8) * 16 +
           4 * (size_t)wide_max_chunk_rows(A->BR) * 8;
}

// the widest compiled tile whose records fit the fetching waves' registers and whose stages fit LDS; 0: none
static int conv_wide_main_tile(const grim_bcr_matrix *A, int KK) {
    for (int tn : {192, 128, 96}) {
        if (A->BR == 32 ? tn != 96 : tn == 96) continue;
        if ((int64_t)A->mmaw.amax[2] <= (int64_t)wide_sru(tn) * kWideFetchThreads && conv_wide_lds(A, tn, KK) <= 160 * 1024) return tn;
    }
    return 0;
}

// Does the layer qualify, and is it large enough for at least one whole round at the widest tile?
bool conv_wide_applies(const grim_bcr_matrix *A, const void *F, int32_t Cin, int32_t H, int32_t W, int32_t kh, int32_t kw,
                       int32_t batch, int64_t f_img_stride, const void *Y, int32_t odt, int64_t ldy, int64_t y_img_stride) {
    if (!A->mmaw.present || A->dtype == GRIM_F32 || (A->BR != 16 && A->BR != 32)) return false;
    if (A->nbr < 8) return false;      // with few strips most multiplying waves idle: the row-gathering kernel is faster
    if (A->mmaw.chunk_rows > wide_max_chunk_rows(A->BR)) return false;
    const int64_t HW = (int64_t)H * W, N = HW * batch;
    const int KK = kh * kw;
    if (HW % 8 != 0 || KK > 255 || A->K * (int64_t)KK >= (int64_t(1) << 31) || HW >= (1 << 24)) return false;
    const int kw_magic = (256 + kw - 1) / kw;
    for (int tap = 0; tap < KK; ++tap)
        if (((tap * kw_magic) >> 8) != tap / kw) return false;
    const int64_t f_total = (batch - 1) * f_img_stride + (int64_t)Cin * HW;
    if (f_total < 8 || f_total * 2 >= (int64_t(1) << 31) || reinterpret_cast<uintptr_t>(F) % 2 != 0) return false;
    // a lane of the 16-row form stores 4 consecutive outputs at once
    if (A->BR == 16 && odt == GRIM_F32 &&
        (reinterpret_cast<uintptr_t>(Y) % 16 != 0 || ldy % 4 != 0 || (batch > 1 && y_img_stride % 4 != 0))) return false;
    const int tn = conv_wide_main_tile(A, KK);
    if (!tn) return false;
    const int64_t groups = (A->nbr + kWideStrips - 1) / kWideStrips;
    const int64_t per_round = 256 / groups;
    return per_round > 0 && N / tn >= per_round;
}

template <bool BF16, int BR, int NT>
static grim_status launch_conv_wide_inst(const WideParams &p, size_t lds, int64_t nwg, hipStream_t stream) {
    auto kern = bcr_spmm_wide<BF16, BR, NT, true>;
    static std::atomic<bool> attr_done{false};
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

// The wide-tile workgroups and, behind them in the same launch, the workgroups of the row-gathering convolution (its
// twelve-wave form, row numbers split in the kernel) for the positions left over: they start on whichever compute unit
// is done with its wide workgroup instead of behind a dispatch of their own.
template <bool BF16, int BR, int NT>
__global__ void __launch_bounds__(kWideThreads) bcr_conv_wide_rest(WideParams wp, ConvParams cp, int wide_wgs) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    if ((int)blockIdx.x < wide_wgs) {
        wide_body<BF16, BR, NT, true>(wp, lds, blockIdx.x);
        return;
    }
    conv_gather_body<BF16, false, kConvLongWaves, 0>(cp, lds, (int)blockIdx.x - wide_wgs);
}
static_assert(kConvLongWaves * 64 == kWideThreads, "the two bodies share the workgroup's twelve waves");

template <bool BF16, int BR, int NT>
static grim_status launch_conv_wide_rest_inst(const WideParams &wp, const ConvParams &cp, size_t lds, int64_t wide_wgs, int64_t rest_wgs,
                                              hipStream_t stream) {
    auto kern = bcr_conv_wide_rest<BF16, BR, NT>;
    static std::atomic<bool> attr_done{false};
    if (lds > 64 * 1024 && !attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) {
            (void)hipGetLastError();
            return GRIM_ERR_DEVICE;
        }
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(wide_wgs + rest_wgs)), dim3(kWideThreads), lds, stream, wp, cp, (int)wide_wgs);
    return hipGetLastError() == hipSuccess ? GRIM_OK : GRIM_ERR_DEVICE;
}

// positions [n_begin, n_end) of the batch in tiles of tn (n_end - n_begin >= tn, both multiples of 8); with `rest`, its
// workgroups (`rest_wgs` of them, `rest_lds` bytes of workgroup memory) behind the wide ones in the same launch
static grim_status conv_wide_range(const grim_bcr_matrix *A, WideParams p, int tn, int64_t n_begin, int64_t n_end, hipStream_t stream,
                                   const ConvParams *rest = nullptr, int64_t rest_wgs = 0, size_t rest_lds = 0) {
    p.n_begin = n_begin;
    p.N = n_end;
    p.ntiles = (int32_t)((n_end - n_begin + tn - 1) / tn);
    const int64_t nwg = ((int64_t)p.ntiles + 15) / 16 * 16 * p.ngroups;
    if (nwg + rest_wgs > 0x7fffffff) return GRIM_ERR_SHAPE;
    if (rest) {
        const size_t lds2 = std::max(conv_wide_lds(A, tn, p.KK), rest_lds);
        if (lds2 > 160 * 1024) return GRIM_ERR_UNSUPPORTED;
        const bool bf2 = A->dtype == GRIM_BF16;
        if (A->BR == 16) {
            if (tn == 192) return bf2 ? launch_conv_wide_rest_inst<true, 16, 12>(p, *rest, lds2, nwg, rest_wgs, stream) : launch_conv_wide_rest_inst<false, 16, 12>(p, *rest, lds2, nwg, rest_wgs, stream);
            if (tn == 128) return bf2 ? launch_conv_wide_rest_inst<true, 16, 8>(p, *rest, lds2, nwg, rest_wgs, stream) : launch_conv_wide_rest_inst<false, 16, 8>(p, *rest, lds2, nwg, rest_wgs, stream);
            return GRIM_ERR_UNSUPPORTED;
        }
        if (tn == 96) return bf2 ? launch_conv_wide_rest_inst<true, 32, 3>(p, *rest, lds2, nwg, rest_wgs, stream) : launch_conv_wide_rest_inst<false, 32, 3>(p, *rest, lds2, nwg, rest_wgs, stream);
        return GRIM_ERR_UNSUPPORTED;
    }
    const size_t lds = conv_wide_lds(A, tn, p.KK);
    const bool bf = A->dtype == GRIM_BF16;
    if (A->BR == 16) {
        if (tn == 192) return bf ? launch_conv_wide_inst<true, 16, 12>(p, lds, nwg, stream) : launch_conv_wide_inst<false, 16, 12>(p, lds, nwg, stream);
        if (tn == 128) return bf ? launch_conv_wide_inst<true, 16, 8>(p, lds, nwg, stream) : launch_conv_wide_inst<false, 16, 8>(p, lds, nwg, stream);
        return bf ? launch_conv_wide_inst<true, 16, 2>(p, lds, nwg, stream) : launch_conv_wide_inst<false, 16, 2>(p, lds, nwg, stream);
    }
    if (tn == 96) return bf ? launch_conv_wide_inst<true, 32, 3>(p, lds, nwg, stream) : launch_conv_wide_inst<false, 32, 3>(p, lds, nwg, stream);
    return bf ? launch_conv_wide_inst<true, 32, 1>(p, lds, nwg, stream) : launch_conv_wide_inst<false, 32, 1>(p, lds, nwg, stream);
}

grim_status launch_conv_wide(const grim_bcr_matrix *A, const void *F, int32_t Cin, int32_t H, int32_t W, int32_t kh,
                             int32_t kw, int32_t batch, int64_t f_img_stride, const float *bias, int32_t relu, void *Y,
                             int32_t odt, int64_t ldy, int64_t y_img_stride, hipStream_t stream) {
    if (!conv_wide_applies(A, F, Cin, H, W, kh, kw, batch, f_img_stride, Y, odt, ldy, y_img_stride)) return GRIM_ERR_UNSUPPORTED;
    const MmaLayout &L = A->mmaw;
    const int64_t HW = (int64_t)H * W, N = HW * batch;
    WideParams p{};
    p.recs = L.d_recs; p.cptr = L.d_cptr; p.bptr = L.d_bptr;
    p.strip_order = A->dev.strip_order;
    p.X = nullptr;
    p.Y = static_cast<float *>(Y);
    p.ldx = 0; p.ldy = ldy;
    p.K = (int32_t)A->K; p.nbr = (int32_t)A->nbr; p.nchunks = L.nchunks; p.chunk_rows = L.chunk_rows;
    p.ngroups = (int32_t)((A->nbr + kWideStrips - 1) / kWideStrips);
    p.amax = L.amax[2];
    p.F = static_cast<const unsigned short *>(F);
    p.H = H; p.W = W; p.HW = (int32_t)HW; p.kh = kh; p.kw = kw; p.KK = kh * kw;
    p.kk_magic = (int32_t)(uint32_t)(((uint64_t(1) << 31) + p.KK - 1) / p.KK);
    p.kw_magic = (256 + kw - 1) / kw;
    p.f_img_stride = (int32_t)(batch > 1 ? f_img_stride : 0);
    p.f_total = (int32_t)((batch - 1) * (int64_t)p.f_img_stride + (int64_t)Cin * HW);
    p.y_img_stride = batch > 1 ? y_img_stride : 0;
    p.bias = bias; p.relu = relu; p.odt = odt;
    const int tn = conv_wide_main_tile(A, p.KK);
    const int64_t per_round = 256 / p.ngroups;
    const int64_t n_main = N / tn / per_round * per_round * tn;
    grim_status st;
    if (n_main == N) return conv_wide_range(A, p, tn, 0, n_main, stream);
    // What is left.  A narrow tile of this kernel walks all K for its 16 strips in one chain of chunk periods whatever
    // its width (16 workgroups: 50 us for the last 512 positions of a 4608-row layer), so a rest of at least 64 positions
    // inside one image goes to the row-gathering convolution, whose workgroups split the strips and K (256 workgroups
    // for the same positions).  Otherwise narrow tiles; fewer than one tile's worth: the last 32 positions, of which the
    // first few are computed twice (the same sums in the same order: the overlap writes the same bits).
    const int64_t img_r = n_main / HW;
    if (N - n_main >= 64 && (N - 1) / HW == img_r && A->gather.present) {
        const char *Fi = static_cast<const char *>(F) + img_r * (int64_t)p.f_img_stride * 2;
        char *Yi = static_cast<char *>(Y) + img_r * p.y_img_stride * (odt == GRIM_F32 ? 4 : 2);
        // in the same launch when the rest takes the form of that kernel the combined kernel carries
        ConvParams cp;
        ConvForm form;
        st = conv_gather_setup(A, Fi, Cin, H, W, kh, kw, bias, relu, Yi, odt, ldy, 1, 1, 0, 0, nullptr, 0, n_main - img_r * HW,
                               N - img_r * HW, &cp, &form);
        if (st == GRIM_OK && !form.solo && form.longw == kConvLongWaves && form.mode == 0) {
            st = conv_wide_range(A, p, tn, 0, n_main, stream, &cp, form.nwg, form.lds);
            if (st != GRIM_ERR_UNSUPPORTED) return st;
        }
        st = conv_wide_range(A, p, tn, 0, n_main, stream);
        if (st != GRIM_OK) return st;
        st = launch_conv_gather(A, Fi, Cin, H, W, kh, kw, bias, relu, Yi, odt, ldy, stream, 1, 1, 0, 0, nullptr, 0,
                                n_main - img_r * HW, N - img_r * HW);
        if (st != GRIM_ERR_UNSUPPORTED) return st;
    } else {
        st = conv_wide_range(A, p, tn, 0, n_main, stream);
        if (st != GRIM_OK) return st;
    }
    const int64_t rest0 = N - n_main >= kConvWideRestTile ? n_main : N - kConvWideRestTile;
    return conv_wide_range(A, p, kConvWideRestTile, rest0, N, stream);
}

}  // namespace grim

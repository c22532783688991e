#include "conv_gather_kernel.hpp"

namespace grim {

// The window-start word of one k slot (row `k` of the im2col matrix, 0xffffffff: padding) for a convolution plan.
uint32_t conv_plan_word(uint32_t k, int32_t H, int32_t W, int32_t kh, int32_t kw) {
    const int32_t KK = kh * kw;
    if (k == 0xffffffffu) return (uint32_t)KK << 27 | (1u << 25);
    const int64_t cin = k / KK;
    const int32_t tap = (int32_t)(k % KK), r = tap / kw, q = tap % kw;
    const int64_t eb = cin * H * W + (int64_t)r * W + q - ((int64_t)(kh / 2) * W + kw / 2);
    return (uint32_t)tap << 27 | (uint32_t)(eb + (1 << 25));
}

grim_status conv_gather_setup(const grim_bcr_matrix *A, const void *F, int32_t Cin, int32_t H, int32_t W, int32_t kh, int32_t kw,
                              const float *bias, int32_t relu, void *Y, int32_t odt, int64_t ldy, int32_t batch, int32_t stride,
                              int64_t f_img_stride, int64_t y_img_stride, const uint32_t *plan, int32_t img0, int64_t pos_begin,
                              int64_t pos_end, ConvParams *out, ConvForm *form) {
    const int64_t N = (int64_t)H * W, total = (int64_t)Cin * N;
    if (batch < 1 || (stride != 1 && stride != 2)) return GRIM_ERR_UNSUPPORTED;
    if (!A->gather.present || total < 8 || kh * kw > kConvMaxTaps || total > (int64_t(1) << 26) || (int64_t)(kh / 2) * W + kw / 2 >= (1 << 24) ||
        A->K > (int64_t(1) << 27) || A->K * (int64_t)(kh * kw) > (int64_t(1) << 31) || Cin >= (1 << 24) || N >= (1 << 24) || reinterpret_cast<uintptr_t>(F) % 2 != 0)
        return GRIM_ERR_UNSUPPORTED;
    ConvParams p;
    p.sptr = A->gather.d_sptr;
    p.out_row = A->gather.d_out_row;
    p.rows = A->gather.d_rows;
    p.desc = A->gather.d_desc;
    p.payload = A->gather.d_payload;
    p.F = static_cast<const unsigned short *>(F);
    p.Y = Y;
    p.bias = bias;
    p.odt = odt;
    p.relu = relu;
    p.ldy = ldy;
    p.N = (int32_t)N; p.H = H; p.W = W; p.kh = kh; p.kw = kw;
    p.KK = kh * kw;
    p.kk_magic = (int32_t)(uint32_t)(((uint64_t(1) << 31) + p.KK - 1) / p.KK);
    p.kw_magic = (256 + kw - 1) / kw;
    for (int tap = 0; tap < p.KK; ++tap)
        if (((tap * p.kw_magic) >> 8) != tap / kw) return GRIM_ERR_UNSUPPORTED;   // (1 x 25 and the like)
    p.total = (int32_t)total;
    p.nbr = (int32_t)A->gather.nstrips;
    p.usteps = A->gather.usteps;
    p.plan = plan;
    p.batch = batch;
    p.f_img_stride = f_img_stride;
    p.y_img_stride = y_img_stride;
    p.stride = stride;
    p.hmul = stride == 2 && W % 8 == 0 ? 2 : 1;
    p.Wo = (W + stride - 1) / stride;
    int64_t Nv = p.hmul == 2 ? (int64_t)((H + 1) / 2) * W : N;
    p.img0 = img0;
    p.pos_begin = 0;
    if (pos_end > 0) {
        // a range of positions of one image (stride 1): at least one tile's worth, so that the ragged last tile stays inside it
        if (stride != 1 || batch != 1 || pos_begin < 0 || pos_end > N || pos_end - pos_begin < 64) return GRIM_ERR_UNSUPPORTED;
        p.pos_begin = (int32_t)pos_begin;
        Nv = pos_end;
    }
    p.Nv = (int32_t)Nv;
    p.tiles_per_img = (int32_t)((Nv - p.pos_begin + 63) / 64);
    if ((int64_t)p.tiles_per_img * batch > 0x7fffffff / 16) return GRIM_ERR_SHAPE;
    p.ntiles = p.tiles_per_img * batch;
    // four consecutive outputs of a row in one store: 16 bytes of fp32, 8 bytes of fp16 / bf16
    const int esz_out = odt == GRIM_F32 ? 4 : 2;
    p.yvec = (stride == 1 && reinterpret_cast<uintptr_t>(Y) % (odt == GRIM_F32 ? 16 : 8) == 0 && ldy % 4 == 0 && N % 4 == 0 &&
              (batch == 1 || (y_img_stride * esz_out) % (odt == GRIM_F32 ? 16 : 8) == 0)) ? 4 : 1;
    // the same launch forms as the row-gathering kernel
    const bool solo = gather_wave_per_strip(A, (int64_t)p.ntiles * p.nbr, 4096);
    const int64_t pairs = (int64_t)p.ntiles * p.nbr;
    // long strips and few pairs: twelve waves per strip up to 256 pairs (one workgroup per compute unit), eight up to 512
    // (two per compute unit; 28 x 28 layers: 11.0 -> 9.4 us with 18 steps, 14.1 -> 13.3 us with 36)
    const int longw = !solo && A->gather.max_steps >= 16 ? (pairs <= 256 ? kConvLongWaves : pairs <= 512 ? 8 : 0) : 0;
    const int64_t per_tile = solo ? (p.nbr + 3) / 4 : p.nbr;
    if (((int64_t)p.ntiles + 7) / 8 * 8 * per_tile > 0x7fffffff) return GRIM_ERR_SHAPE;
    int64_t nwg = 0;
    p.map = xcd_map(p.ntiles, per_tile, &nwg);
    if (nwg > 0x7fffffff) return GRIM_ERR_SHAPE;
    if (stride == 2 && !plan) return GRIM_ERR_UNSUPPORTED;
    form->solo = solo;
    form->longw = longw;
    form->mode = stride == 2 ? 2 : plan ? 1 : 0;
    form->nwg = nwg;
    form->lds = (size_t)(longw ? longw : 4) * 8192 + kConvTableBytes;
    *out = p;
    return GRIM_OK;
}

grim_status launch_conv_gather(const grim_bcr_matrix *A, const void *F, int32_t Cin, int32_t H, int32_t W, int32_t kh,
                               int32_t kw, const float *bias, int32_t relu, void *Y, int32_t odt, int64_t ldy,
                               hipStream_t stream, int32_t batch, int32_t stride, int64_t f_img_stride,
                               int64_t y_img_stride, const uint32_t *plan, int32_t img0, int64_t pos_begin, int64_t pos_end) {
    ConvParams p;
    ConvForm form;
    const grim_status st = conv_gather_setup(A, F, Cin, H, W, kh, kw, bias, relu, Y, odt, ldy, batch, stride, f_img_stride,
                                             y_img_stride, plan, img0, pos_begin, pos_end, &p, &form);
    if (st != GRIM_OK) return st;
    const bool solo = form.solo;
    const int longw = form.longw, mode = form.mode;
    const size_t lds = form.lds;
    const dim3 grid((unsigned)form.nwg), block(longw ? longw * 64 : 256);
#define GRIM_CONV_M(BF, SO, EI, MO)                                                                                  \
    do {                                                                                                             \
        auto kern = bcr_conv_gather<BF, SO, EI, MO>;                                                                 \
        static std::atomic<bool> attr_done{false};                                                                   \
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
#define GRIM_CONV(BF, SO, EI)                                                                                        \
    do {                                                                                                             \
        if (mode == 0) GRIM_CONV_M(BF, SO, EI, 0); else if (mode == 1) GRIM_CONV_M(BF, SO, EI, 1); else GRIM_CONV_M(BF, SO, EI, 2); \
    } while (0)
    if (A->dtype == GRIM_BF16) { if (solo) GRIM_CONV(true, true, 0); else if (longw == 12) GRIM_CONV(true, false, 12); else if (longw == 8) GRIM_CONV(true, false, 8); else GRIM_CONV(true, false, 0); }
    else { if (solo) GRIM_CONV(false, true, 0); else if (longw == 12) GRIM_CONV(false, false, 12); else if (longw == 8) GRIM_CONV(false, false, 8); else GRIM_CONV(false, false, 0); }
#undef GRIM_CONV
#undef GRIM_CONV_M
    return hipGetLastError() == hipSuccess ? GRIM_OK : GRIM_ERR_DEVICE;
}


}  // namespace grim

// Internal definitions shared by the host packer and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>
#include <vector>

#include "grim_bcr.h"

namespace grim {

constexpr int kMmaMaxChunkRows = 256;   // rows of X staged in LDS per step by the matrix-core kernel
// the same for the wide-tile kernel: 128 rows of its 128- and 192-column tiles (BR = 16), 192 rows of its 96-column
// tiles (BR = 32) -- what two LDS stages hold
constexpr int wide_max_chunk_rows(int BR) { return BR == 32 ? 192 : 128; }
constexpr int kWideMaxRecordBytes = 32 * 1024;   // records of one (chunk, group of 16 strips) the wide-tile kernel stages
constexpr int kGemvMaxXBytes = 65536;   // bytes of x (K * batch elements) the SpMV kernel keeps in LDS

inline int dtype_size(int dt) { return dt == GRIM_F32 ? 4 : 2; }

// Layout for the matrix-core SpMM kernel (fp16 / bf16, BR = 16 or 32).
// K is cut into chunks of `chunk_rows` consecutive rows of X.  For every (chunk, stored strip)
// the kept columns of the strip's blocks inside the chunk are laid out as groups of 8 k slots
// (a block's columns are padded to a multiple of 8 with the all-zero staged row), `ks / 8`
// groups per MFMA step.  A (chunk, strip) region is
//   [steps x header][payload]
//   header : per step, the staged-row numbers of its k slots (u16, ordered so that the pair a
//            lane names in its two LDS transpose reads is adjacent), then per group the block's
//            row bit mask (u32) and the offset of the group's weights in 16-byte units from the
//            region start (u32);
//   payload: per group, for every KEPT row of the block 8 weights (16 bytes) -- compact: pruned
//            rows are not stored; a lane finds its row by popcount of the mask below its bit.
// Regions are stored chunk-major, strips in stored order inside a chunk, so what a workgroup
// (a group of consecutive stored strips) needs for one chunk is one contiguous byte range.
struct MmaLayout {
    bool present = false;
    int32_t ks = 0;            // 32 for BR = 16 (16x16x32), 16 for BR = 32 (32x32x16)
    int32_t chunk_blocks = 0;  // column blocks per chunk
    int32_t chunk_rows = 0;    // chunk_blocks * BC
    int32_t nchunks = 0;
    int64_t nsteps = 0;
    int32_t amax[4] = {0, 0, 0, 0};   // most 16-byte units any (group, chunk) holds, for groups of 4, 8, 16, 32 strips
    std::vector<int32_t> cptr;        // [nchunks * (nbr + 1)] first step of (chunk, stored strip); last = end of chunk
    std::vector<int32_t> bptr;        // same shape: region start in 16-byte units
    std::vector<unsigned char> recs;
    int32_t *d_cptr = nullptr;
    int32_t *d_bptr = nullptr;
    unsigned char *d_recs = nullptr;
    int64_t bytes = 0;
};

// Layout for the row-gathering matrix-core SpMM kernel (fp16 / bf16; block heights that divide 16
// or are multiples of 16).  The rows of the matrix in stored order (stored strip p, local row r ->
// p * BR + r) are cut into runs of 16, the MFMA tile height: a run is one strip for BR = 16, a
// quarter of a strip for BR = 64, four strips for BR = 4.  The kept columns of the blocks that
// reach into a run, in column-block order, are cut into groups of 8 k slots (a block's columns
// padded to a multiple of 8; a group belongs to one block and carries that block's kept rows
// inside the run as a 16-bit mask) and groups into steps of 32 k slots -- one v_mfma_f32_16x16x32
// per 16 columns of X.  Nothing depends on how K is cut: a wave takes any contiguous range of a
// run's steps.
//   rows   : per step 32 x u32, the row of X behind k slot g * 8 + j at position j * 4 + g
//            (0xffffffff = padding: the slot multiplies zeros), so that the lane that fetches slots
//            j, j + 8, j + 16, j + 24 reads its four row numbers with one 16-byte load;
//   desc   : per step and group the block's row bit mask (u32) and the place of the group's
//            weights in `payload`, in 16-byte units (u32);
//   payload: per group, for every KEPT row of the block 8 weights (16 bytes).
struct GatherLayout {
    bool present = false;
    int64_t nsteps = 0;
    int64_t xrows = 0;                    // k slots that name a row of X (not padding), over all strips
    int64_t nstrips = 0;                  // 16-row runs: ceil(M / 16)
    int32_t usteps = 0;                   // > 0: every run has this many steps (the kernels then skip the sptr look-up)
    int32_t max_steps = 0;                // most steps any run has
    std::vector<int32_t> sptr;            // [nstrips + 1] first step of each run
    std::vector<int32_t> out_row;         // [nstrips * 16] original row of every stored row (-1 past M)
    std::vector<uint32_t> rows;           // [nsteps * 32]
    std::vector<uint32_t> desc;           // [nsteps * 8]
    std::vector<unsigned char> payload;
    int32_t *d_sptr = nullptr;
    int32_t *d_out_row = nullptr;
    uint32_t *d_rows = nullptr;
    uint32_t *d_desc = nullptr;
    unsigned char *d_payload = nullptr;
    int64_t bytes = 0;
};

// Layout for the SpMV kernel (BR, BC <= 32): the compact weights themselves plus one
// row bit mask and one column bit mask per stored block.
struct GemvLayout {
    bool present = false;
    int32_t uniform_kr = -1, uniform_kc = -1;   // >= 0 when every block keeps the same counts
    int32_t vec = 1;                            // widest aligned vector (elements) for weight rows
    int32_t krmax = 0, kcmax = 0;               // most rows / columns any block keeps
    std::vector<uint32_t> masks;                // [nb * 2] (rowmask, colmask)
    std::vector<uint32_t> woff;                 // [nb + 1] element offsets (32-bit copy of blk_ptr)
    uint32_t *d_masks = nullptr;
    uint32_t *d_woff = nullptr;
    int64_t bytes = 0;
};

struct DeviceCanonical {
    int32_t *strip_order = nullptr;
    int32_t *strip_pos = nullptr;    // inverse of strip_order: stored position of original strip s
    int32_t *row_ptr = nullptr;
    uint16_t *row_idx = nullptr;
    int32_t *col_ptr = nullptr;
    uint16_t *col_idx = nullptr;
    int64_t *blk_ptr = nullptr;
    void *weights = nullptr;
    uint64_t *rowmask64 = nullptr;   // per stored block, bit r set when local row r is kept (BR <= 64)
    int64_t bytes = 0;
};

}  // namespace grim

struct grim_bcr_matrix {
    int64_t M = 0, K = 0;
    int32_t BR = 0, BC = 0;
    int32_t dtype = 0;
    int32_t reordered = 0;
    int64_t nbr = 0, nbc = 0, nb = 0, nnz = 0;
    // canonical host arrays (stored order)
    std::vector<int32_t> strip_order;
    bool order_identity = false;     // stored strip p is original strip p (equal work everywhere: the stable sort moved nothing)
    std::vector<int32_t> row_ptr, col_ptr;
    std::vector<uint16_t> row_idx, col_idx;
    std::vector<int64_t> blk_ptr;
    std::vector<unsigned char> weights;
    std::vector<uint64_t> rowmask64;
    // device side
    bool on_device = false;
    int device = -1;
    grim::DeviceCanonical dev;
    grim::MmaLayout mma;
    grim::MmaLayout mmaw;   // the same records cut for chunks of at most 128 rows (wide-tile kernel)
    grim::GatherLayout gather;
    grim::GemvLayout gemv;
    // exchange words of the whole-sequence recurrent kernel (2 x H x 8 bytes), allocated by the first such call
    mutable void *seq_exch = nullptr;
    mutable std::mutex seq_lock;
};

// The paper's six BCRC arrays (Section 4.3), host side.
struct grim_bcrc {
    int64_t M = 0, K = 0;
    int32_t dtype = 0;
    std::vector<int32_t> reorder;
    std::vector<int64_t> row_offset;
    std::vector<int32_t> occurrence;
    std::vector<int64_t> column_stride;
    std::vector<int32_t> compact_column;
    std::vector<unsigned char> weights;
};

// Descriptor of one matrix as the SpMV kernel reads it (device table entry of a group).
struct GemvDesc {
    const void *weights;
    const uint32_t *masks;
    const uint32_t *woff;
    const int32_t *strip_order;
};

// Recurrent cell applied in the epilogue of the one-right-hand-side wave-per-strip kernel (Section 3.1: an RNN layer
// is one matrix-vector product per time step; the gate nonlinearities and the state update are the elementwise rest).
// A workgroup then owns BR hidden units: its waves take the strips that hold these units' gate rows -- LSTM: four
// strips of [W_ih | W_hh] (input, forget, candidate, output gate); GRU: three strips (reset, update, candidate) of
// each of W_i and W_h -- found through `strip_pos`, the stored position of every original strip.
struct RnnCell {
    const int32_t *strip_pos;    // first matrix: stored position of original strip s; nullptr: strip s is stored at s
    const int32_t *strip_pos2;   // second matrix (GRU)
    const float *bias, *bias2;   // LSTM: 4H (bias); GRU: 3H input side (bias), 3H hidden side (bias2); null = none
    float *c;                    // LSTM: cell state, H fp32, stride ldc, updated in place; GRU: hidden state h32
    void *h;                     // new hidden state in element type hdt, stride ldh (null: not written)
    float *h32;                  // LSTM: optional fp32 copy of the new hidden state, stride ldh32
    int64_t ldc, ldh, ldh32;
    int32_t H, hdt;
};

struct grim_bcr_group {
    int32_t count = 0;
    int64_t M = 0, K = 0;
    int32_t BR = 0, BC = 0, dtype = 0;
    int64_t nbr = 0, nbc = 0;
    int32_t uniform_kr = -1, uniform_kc = -1, vec = 1, krmax = 0, kcmax = 0;
    int device = -1;
    GemvDesc *d_table = nullptr;
};

namespace grim {
// kernel launchers (defined in the .hip files); all enqueue on `stream` and return a status
grim_status launch_spmm_fma(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, float *Y,
                            int64_t ldy, hipStream_t stream);
grim_status launch_spmm_mma(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, float *Y,
                            int64_t ldy, int32_t tile_n, int32_t strips_per_wg, hipStream_t stream);
bool mma_supported(const grim_bcr_matrix *A);
// wide-tile staged kernel: tile_n 0 = choose; wide_applies: operands and matrix qualify for some tile width
grim_status launch_spmm_wide(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, float *Y, int64_t ldy,
                             int32_t tile_n, hipStream_t stream);
// the same with the columns from wide_cols on computed by row-gathering workgroups in the same launch; UNSUPPORTED
// (nothing enqueued) when those columns do not take the form of that kernel the launch is built for
grim_status launch_spmm_wide_with_rest(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, float *Y, int64_t ldy,
                                       int32_t tile_n, int64_t wide_cols, hipStream_t stream);
bool wide_applies(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, const float *Y, int64_t ldy, int32_t tile_n);
// best use of the wide-tile kernel: cost (bytes through one compute unit; < 0: does not apply), tile width and the
// leading columns it should take (N, or whole rounds of workgroups with the rest priced by rest_cost)
double wide_plan(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, const float *Y, int64_t ldy,
                 double (*rest_cost)(const grim_bcr_matrix *, int64_t), int *tn_out, int64_t *n_main);
// row-gathering matrix-core kernel; GRIM_ERR_UNSUPPORTED when the matrix or the operands do not qualify
// A2 / X2 / Y2: a second product of the same N, ldx and ldy in the same launch (gather_pair_applies)
grim_status launch_spmm_gather(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx, float *Y,
                               int64_t ldy, hipStream_t stream, const grim_bcr_matrix *A2 = nullptr,
                               const void *X2 = nullptr, float *Y2 = nullptr);
bool gather_pair_applies(const grim_bcr_matrix *A, const void *X, const grim_bcr_matrix *A2, const void *X2, int64_t N,
                         int64_t ldx);
bool gather_applies(const grim_bcr_matrix *A, const void *X, int64_t N, int64_t ldx);
// launch form of the row-gathering kernels: a (tile, strip) pair per wave instead of four waves per strip
bool gather_wave_per_strip(const grim_bcr_matrix *A, int64_t pairs, int64_t pairs_for_long_strips);
// convolution on the row-gathering layout, the im2col matrix never formed
// batch images f_img_stride / y_img_stride elements apart; stride 1 or 2 ("same" padding, output ceil(H / stride) x
// ceil(W / stride)); plan: the k slots' window-start words (conv_plan_word) on the device, or null
grim_status launch_conv_gather(const grim_bcr_matrix *A, const void *F, int32_t Cin, int32_t H, int32_t W, int32_t kh,
                               int32_t kw, const float *bias, int32_t relu, void *Y, int32_t odt, int64_t ldy,
                               hipStream_t stream, int32_t batch = 1, int32_t stride = 1, int64_t f_img_stride = 0,
                               int64_t y_img_stride = 0, const uint32_t *plan = nullptr, int32_t img0 = 0,
                               int64_t pos_begin = 0, int64_t pos_end = 0);   // pos_end > 0: positions [pos_begin, pos_end) of image img0 only
uint32_t conv_plan_word(uint32_t k, int32_t H, int32_t W, int32_t kh, int32_t kw);
// stride-1 convolution of layers with many positions on the wide-tile kernel (whole rounds of workgroups plus a narrow
// rest); GRIM_ERR_UNSUPPORTED when the layer is too small or does not qualify: the caller then takes the kernel above
bool conv_wide_applies(const grim_bcr_matrix *A, const void *F, int32_t Cin, int32_t H, int32_t W, int32_t kh, int32_t kw,
                       int32_t batch, int64_t f_img_stride, const void *Y, int32_t odt, int64_t ldy, int64_t y_img_stride);
grim_status launch_conv_wide(const grim_bcr_matrix *A, const void *F, int32_t Cin, int32_t H, int32_t W, int32_t kh,
                             int32_t kw, int32_t batch, int64_t f_img_stride, const float *bias, int32_t relu, void *Y,
                             int32_t odt, int64_t ldy, int64_t y_img_stride, hipStream_t stream);
// cost estimates (bytes through one compute unit) used to choose between the two matrix-core kernels
double gather_cost(const grim_bcr_matrix *A, int64_t N);
double mma_best_shape(const grim_bcr_matrix *A, int64_t N, int32_t tile_n, int32_t strips_per_wg, int *tn_out, int *g_out);
int64_t mma_whole_rounds(const grim_bcr_matrix *A, int64_t N, bool rest_may_gather, int *tn_out, int *g_out);
// matrices of one launch: a device table of `count` descriptors, or (no table) `single` alone, or
// `single` and `*second` (count = 2)
grim_status launch_spmv(const GemvDesc *table_dev_or_null, const GemvDesc &single, const GemvDesc *second, int32_t count,
                        int64_t M, int64_t K, int32_t BR, int32_t BC, int32_t dtype, int32_t ukr,
                        int32_t ukc, int32_t vec, int32_t krmax, int32_t kcmax, const void *x, int64_t x_stride, int32_t batch,
                        int64_t ldx, float *y, int64_t y_stride, int64_t ldy, hipStream_t stream);
bool spmv_cell_applies(int kind, int64_t M, int64_t K, int32_t BR, int32_t BC, int32_t dtype, int32_t ukr, int32_t ukc, int64_t H);
// a recurrent step in one launch: the product(s) with the cell in the epilogue, one set of workgroups per column of x
constexpr int32_t kCellMaxBatch = 32;
bool spmv_cell_batch_ok(int64_t H, int32_t BR, int32_t batch);   // all sets of workgroups in one round on this GPU?
bool spmv_exact_applies(int32_t dtype, int32_t ukr, int32_t ukc, int64_t K);
bool spmv_column_sets_ok(int64_t count, int64_t nbr, int32_t batch);   // columns as sets of workgroups of the one-column kernel
grim_status launch_spmv_cell(int kind, const GemvDesc &d1, const GemvDesc *d2, int64_t M, int64_t K, int32_t BR, int32_t BC,
                             int32_t dtype, int32_t ukr, int32_t ukc, const void *x, int64_t x_stride, int32_t batch, int64_t ldx,
                             float *y, int64_t y_stride, int64_t ldy, const RnnCell &cell, hipStream_t stream);
// a recurrent layer over a whole sequence in one launch (kind 1: LSTM, K1 = I + H; kind 2: GRU, K1 = I, K2 = H), `batch`
// sequences side by side (1 .. kSeqMaxBatch); exch: at most 2 * batch * H words of 8 bytes; hidden sizes up to kSeqMaxH
constexpr int64_t kSeqMaxH = 8192;
constexpr int32_t kSeqMaxBatch = 32;
bool rnn_seq_applies(int kind, int32_t BR, int32_t BC, int32_t dtype, int32_t ukr, int32_t ukc, int64_t K1, int64_t K2,
                     int64_t I, int64_t H, int32_t batch);
grim_status launch_rnn_seq(int kind, const GemvDesc &d1, const GemvDesc *d2, const int32_t *pos1, const int32_t *pos2,
                           int32_t BR, int32_t BC, int32_t dtype, int32_t ukr, int32_t ukc, int64_t K1, int64_t K2, int64_t I,
                           int64_t H, int32_t T, int32_t batch, const void *xs, int64_t ldxs, const void *h0, const float *bias,
                           const float *bias2, float *state, void *hs, int64_t ldhs, float *hs32, int64_t ldhs32,
                           void *exch, int32_t *status, uint32_t max_polls, hipStream_t stream);
// device address of this GPU's static exchange words (2 * kSeqMaxH of them); allocates nothing
grim_status rnn_seq_static_exchange(void **out);
grim_status launch_lstm_cell(const float *gates, int64_t ldg, const float *bias, float *c, int64_t ldc, void *h,
                             int32_t dtype, int64_t ldh, float *h32, int64_t ldh32, int64_t H, int32_t batch,
                             hipStream_t stream);
grim_status launch_gru_cell(const float *gi, int64_t ldgi, const float *gh, int64_t ldgh, const float *bias_i,
                            const float *bias_h, float *h32, int64_t ldh32, void *h, int32_t dtype, int64_t ldh,
                            int64_t H, int32_t batch, hipStream_t stream);
}  // namespace grim

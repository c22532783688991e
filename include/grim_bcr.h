/*
 * grim_bcr.h -- C ABI of the BCR (Block-based Column-Row) sparse product library
 * for AMD MI355X (gfx950).
 *
 * The library computes  Y = W_bcr * X : the product of a BCR-pruned weight matrix
 * with dense activations.  This is the inference hot path of GRIM (arXiv 2108.11033):
 *   - Section 3.1 (unified view): CONV layers become weight matrix x im2col input
 *     matrix (SpMM); FC / RNN gate layers become matrix x vector (SpMV).
 *   - Section 3.2 (BCR sparsity): W (M x K) is cut into equal BR x BC blocks
 *     (BR rows = outputs, BC columns = inputs); each block independently keeps a
 *     set of whole rows and a set of whole columns; the survivors of a block form
 *     a full (kept rows) x (kept columns) matrix.  Every other weight is zero.
 *   - Section 4.2 (matrix reorder) and 4.3 (compact storage): rows with the same
 *     amount of work are stored together and zero weights are not stored; the
 *     column indices shared by the rows of a block are stored once.
 *
 * All functions return a grim_status and never throw or abort.  Unless stated
 * otherwise, pointers named *_host are host memory and *_dev are device memory
 * on the GPU that was current when the matrix was packed.  The library never
 * takes ownership of caller memory.
 *
 * Threads: a packed matrix is immutable; any number of threads may launch products of the
 * same matrix on streams of their own (kernels write only the caller's outputs, and there is
 * no workspace shared between calls).  Calls that create or free a handle must not run at
 * the same time as any other call that uses that handle.
 */
#ifndef GRIM_BCR_H
#define GRIM_BCR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct grim_bcr_matrix grim_bcr_matrix; /* opaque; owns its host and device copies */
typedef struct grim_bcr_group grim_bcr_group;   /* opaque; a set of matrices for one batched launch */

typedef enum {
    GRIM_OK = 0,
    GRIM_ERR_NULL = 1,        /* a required pointer is NULL */
    GRIM_ERR_SHAPE = 2,       /* BR does not divide M, BC does not divide K, N < 1, leading
                                 dimension too small, batch outside 1..8, size over a limit */
    GRIM_ERR_INDEX = 3,       /* a ptr array is not monotone / does not start at 0, an index is
                                 out of range, or a block's indices are not strictly ascending */
    GRIM_ERR_DTYPE = 4,       /* unknown grim_dtype */
    GRIM_ERR_ALLOC = 5,       /* host or device allocation failed */
    GRIM_ERR_DEVICE = 6,      /* a HIP call failed, no GPU, or the matrix was packed host-only */
    GRIM_ERR_UNSUPPORTED = 7  /* valid request that no kernel covers (e.g. BR > 64) */
} grim_status;

typedef enum { GRIM_F32 = 0, GRIM_F16 = 1, GRIM_BF16 = 2 } grim_dtype;

/* Options of grim_bcr_pack.  Zero-initialise, then set what differs. */
typedef struct grim_bcr_options {
    int32_t no_reorder;  /* 0 (default): store row strips by decreasing work (Section 4.2);
                            1: keep the natural strip order */
    int32_t host_only;   /* 1: build only the canonical host arrays (pack / unpack / arrays work without
                            a GPU; spmm / spmv then return GRIM_ERR_DEVICE); 2: also build the derived
                            kernel layouts on the host (grim_bcr_unpack_layout), still without a GPU */
    int32_t chunk_rows;  /* rows of X staged per step by the matrix-core SpMM kernel;
                            0 = choose.  Rounded to a whole number of column blocks. */
    int32_t reserved[5];
} grim_bcr_options;

/* Borrowed, read-only view of the canonical compact arrays (host memory owned by
 * the matrix, valid until grim_bcr_free).  "Stored order" of blocks: strips in
 * strip_order, inside a strip column blocks ascending; t = position in that order.
 *   strip_order[nbr]  strips by decreasing work w_s = sum_c kr*kc, ties by index
 *   row_ptr[nb+1], row_idx[]  kept rows of stored block t, local, ascending
 *   col_ptr[nb+1], col_idx[]  kept columns likewise
 *   blk_ptr[nb+1]     offset of stored block t in weights (prefix sums of kr*kc)
 *   weights[nnz]      each block row-major [kept row][kept col]; bit copies of W */
typedef struct grim_bcr_view {
    int64_t M, K;
    int32_t BR, BC;
    int32_t dtype;
    int32_t reordered;
    int64_t nbr, nbc, nb, nnz;
    const int32_t *strip_order;
    const int32_t *row_ptr;
    const uint16_t *row_idx;
    const int32_t *col_ptr;
    const uint16_t *col_idx;
    const int64_t *blk_ptr;
    const void *weights;
    /* bytes of the device-side layouts derived from the arrays above (0 if absent) */
    int64_t dev_bytes_canonical; /* the arrays above, as uploaded */
    int64_t dev_bytes_mma;       /* matrix-core layout: per-step gather lists, row masks and kept-row weights */
    int64_t dev_bytes_gemv;      /* per-block row/column bit masks + offsets for the SpMV kernel */
} grim_bcr_view;

/*
 * grim_bcr_pack -- compact a dense matrix under a BCR mask (Sections 3.2, 4.2, 4.3).
 *   W_host   dense M x K matrix, row-major with leading dimension ldw (elements),
 *            element type dt.  Values at pruned positions are ignored.
 *   BR, BC   block size; BR must divide M and BC must divide K (the paper's block
 *            sizes divide the layer's height and width, Section 5.1).  1 <= BR,BC <= 65535.
 *   row_ptr  nb+1 prefix sums (nb = (M/BR)*(K/BC), blocks numbered b = s*(K/BC) + c);
 *   row_idx  kept rows of block b = row_idx[row_ptr[b] .. row_ptr[b+1]), local to the
 *            block (0..BR-1), strictly ascending.  col_ptr / col_idx likewise (0..BC-1).
 *            A block may keep no rows or no columns (it then stores nothing).
 *   opt      NULL = defaults.
 *   out      receives the new matrix; release with grim_bcr_free.
 * Packing is driven by the index sets only, never by inspecting values: kept weights
 * are bit copies (zeros, negative zeros, NaNs included).  The inputs are copied; the
 * caller may free them on return.  Unless opt->host_only, the device layouts are
 * allocated and uploaded to the current GPU before returning (synchronous).
 * Errors: NULL, SHAPE, INDEX, DTYPE, ALLOC, DEVICE.  On error *out is NULL.
 */
grim_status grim_bcr_pack(const void *W_host, grim_dtype dt, int64_t M, int64_t K, int64_t ldw,
                          int32_t BR, int32_t BC,
                          const int32_t *row_ptr, const uint16_t *row_idx,
                          const int32_t *col_ptr, const uint16_t *col_idx,
                          const grim_bcr_options *opt, grim_bcr_matrix **out);

/* grim_bcr_unpack -- inverse of pack: writes the masked dense M x K matrix (leading
 * dimension ldw >= K, element type of the matrix) to host memory; pruned positions
 * become +0.  Bit-exact with respect to the packed input. */
grim_status grim_bcr_unpack(const grim_bcr_matrix *A, void *W_host_out, int64_t ldw);

/* grim_bcr_unpack_layout -- decode one of the layouts the kernels read (all derived from the compact
 * arrays of Section 4.3 when the matrix is packed) back into the masked dense M x K matrix, exactly as
 * grim_bcr_unpack does from the canonical arrays: a host-side check that a kernel layout holds every kept
 * weight at the row and column the kernel will use it for, and nothing else.
 *   layout  1 = staged matrix-core SpMM (step records per chunk and strip), 2 = row-gathering matrix-core
 *           SpMM / convolution (steps per 16-row run), 3 = SpMV (compact weights + row / column bit masks),
 *           4 = wide-tile staged matrix-core SpMM (the records of 1 cut for chunks of at most 128 rows)
 * Works on any matrix whose layouts were built (host_only 0 or 2).  Errors: NULL, SHAPE (ldw < K, unknown
 * layout), UNSUPPORTED (the matrix has no such layout), INDEX (a layout entry points outside the matrix). */
grim_status grim_bcr_unpack_layout(const grim_bcr_matrix *A, int32_t layout, void *W_host_out, int64_t ldw);

/* grim_bcr_arrays -- fill *v with borrowed pointers to the canonical arrays. */
grim_status grim_bcr_arrays(const grim_bcr_matrix *A, grim_bcr_view *v);

/*
 * grim_bcr_spmm -- Y = W_bcr * X on the GPU (Section 3.1: CONV as GEMM on the im2col
 * matrix; Section 4.2-4.4: compact weights, input rows of a block loaded once and
 * reused by all of its kept rows).
 *   X_dev  K x N, row-major, leading dimension ldx >= N (elements), element type of A.
 *   Y_dev  M x N fp32, row-major, leading dimension ldy >= N, in the ORIGINAL row order.
 *          Overwritten (no accumulation into Y; rows kept by no block are written as 0).
 *   hip_stream  a hipStream_t (NULL = the default stream).  The call only enqueues work:
 *          it never synchronises and never allocates.
 * Accumulation is in fp32 in a fixed order (no atomics): results are bit-reproducible
 * from run to run.  N <= 8 is forwarded to the SpMV kernel when that path supports A.
 * A large product may be enqueued as two kernels on disjoint column ranges (the columns that
 * fill whole rounds of workgroups on a wide-tile kernel, then the rest).
 * Errors: NULL, SHAPE (N < 1, ld too small), DEVICE, UNSUPPORTED.  Argument errors are found before anything is
 * enqueued and leave Y untouched; a launch that the runtime rejects (DEVICE) may follow a first kernel that is
 * already enqueued on its column range.
 */
grim_status grim_bcr_spmm(const grim_bcr_matrix *A, const void *X_dev, int64_t N, int64_t ldx,
                          float *Y_dev, int64_t ldy, void *hip_stream);

/* grim_bcr_spmm_tuned -- grim_bcr_spmm with explicit launch parameters (the paper tunes
 * tile sizes per kernel, Section 4.5; here a handful of choices replaces the search):
 *   tile_n         columns of X per workgroup (32, 64 or 128; with kernel 4: 96 for BR = 32, 128 or 192 for BR = 16;
 *                  0 = choose)
 *   strips_per_wg  row strips per workgroup (4, 8 or 16; 0 = choose)
 *   kernel         0 = choose, 1 = force the portable FMA kernel, 2 = force the staged matrix-core
 *                  kernel (fp16 / bf16, BR = 16 or 32; tile_n / strips_per_wg apply to it),
 *                  3 = force the row-gathering matrix-core kernel (fp16 / bf16, BR a divisor or a
 *                  multiple of 16 -- the paper's 4 x 16 blocks included --, N and ldx multiples of 4,
 *                  X 8-byte aligned; tile_n and strips_per_wg must be 0),
 *                  4 = force the wide-tile staged matrix-core kernel on all N columns (fp16 / bf16, BR = 16 or 32,
 *                  N >= tile_n and a multiple of 8, ldx a multiple of 8, ldy of 4, X and Y 16-byte aligned;
 *                  strips_per_wg must be 0)
 * Combinations that are not compiled, that the matrix or the operands do not qualify for, or whose
 * staging buffers do not fit the 160 KB of LDS for this matrix, return GRIM_ERR_UNSUPPORTED. */
grim_status grim_bcr_spmm_tuned(const grim_bcr_matrix *A, const void *X_dev, int64_t N, int64_t ldx,
                                float *Y_dev, int64_t ldy, int32_t tile_n, int32_t strips_per_wg,
                                int32_t kernel, void *hip_stream);

/* grim_bcr_spmm_kernel_name -- which kernel family the grim_bcr_spmm_tuned call with these arguments
 * would launch: "bcr_spmm_wide" (first launch of a large
 * product), "bcr_spmm_gather", "bcr_spmm_mma" (staged), "bcr_spmm_fma", "bcr_spmv" (N <= 8, but see grim_bcr_spmv), or
 * "none" when the call would fail.  A static string; launches nothing.  For profiling and reports. */
const char *grim_bcr_spmm_kernel_name(const grim_bcr_matrix *A, const void *X_dev, int64_t N, int64_t ldx,
                                      int32_t tile_n, int32_t strips_per_wg, int32_t kernel);

/*
 * grim_bcr_spmv -- y = W_bcr * x for 1..8 right-hand sides (Section 3.1: FC and RNN
 * gate matrices are matrix-vector products).  Same conventions as grim_bcr_spmm with
 * N = batch: x_dev is K x batch (ldx >= batch), y_dev is M x batch fp32 (ldy >= batch).
 * Reads the compact weights exactly once; the bytes moved are the stored weights plus
 * 8 bytes of row/column bit masks per block.  One case runs on the matrix cores instead, as
 * one padded tile of the row-gathering SpMM kernel, because that is quicker: batch = 8 of an
 * fp16 / bf16 matrix that kernel takes, with ldx a multiple of 8 and x_dev 16-byte aligned
 * (grim_bcr_spmm with N = 8 makes the same choice; grim_bcr_spmm_kernel_name reports it).
 * Errors: as grim_bcr_spmm; batch outside 1..8 is GRIM_ERR_SHAPE.
 */
grim_status grim_bcr_spmv(const grim_bcr_matrix *A, const void *x_dev, int32_t batch, int64_t ldx,
                          float *y_dev, int64_t ldy, void *hip_stream);

/*
 * Batched SpMV: many independent (W_i, x_i) products in ONE launch.  A single
 * gate-matrix product moves ~2 MB, far less than a kernel launch costs, so
 * independent products are grouped to fill the GPU.
 * grim_bcr_group_create copies the device descriptors of `count` packed matrices
 * (same M, K, BR, BC, dtype; all packed on the current GPU; 1 <= count <= 65535, one
 * grid row per matrix) into one device table.
 * The matrices must outlive the group.
 * grim_bcr_spmv_batched computes y_i = W_i * x_i for i in [0, count): x_i starts at
 * x_dev + i * x_stride elements (K x batch, ldx), y_i at y_dev + i * y_stride floats.
 */
grim_status grim_bcr_group_create(const grim_bcr_matrix *const *mats, int32_t count,
                                  grim_bcr_group **out);
grim_status grim_bcr_spmv_batched(const grim_bcr_group *G, const void *x_dev, int64_t x_stride,
                                  int32_t batch, int64_t ldx, float *y_dev, int64_t y_stride,
                                  int64_t ldy, void *hip_stream);
void grim_bcr_group_free(grim_bcr_group *G);

/*
 * grim_bcr_conv2d -- a CONV layer without its im2col matrix (Section 3.1: CONV = filter matrix x im2col
 * matrix; Section 4.5: rows of that matrix whose weights are all pruned are skipped).  Stride 1, zero
 * padding kh/2 and kw/2 ("same"), kh and kw odd, batch 1:
 *     Y[m][h * W + w] = sum over (cin, r, q) of W_bcr[m][cin * kh * kw + r * kw + q] *
 *                       F[cin][h + r - kh/2][w + q - kw/2]            (F = 0 outside the image)
 * i.e. column k of the packed matrix is (cin, r, q) in that order (the order of the usual
 * weight.reshape(Cout, Cin * kh * kw)); A must have K = Cin * kh * kw columns.
 *   F_dev  Cin x H x W contiguous, element type of A (any element alignment)
 *   Y_dev  M x (H * W) fp32, leading dimension ldy >= H * W, overwritten
 * The result equals grim_bcr_spmm on the materialised im2col matrix (bit for bit when every sum is
 * exact); only the feature map is read -- kh * kw times fewer bytes -- and only the rows a strip keeps.
 * Runs on the row-gathering matrix-core kernel: fp16 / bf16, block height a divisor or a multiple of
 * 16, H * W < 2^24 (maps of any shape down to 1 x 1: fewer than 64 positions run as one partly
 * filled tile), kh * kw <= 31 (5 x 5, 3 x 7; a few flat shapes such as 1 x 25 are refused),
 * 8 <= Cin * H * W <= 2^26; otherwise GRIM_ERR_UNSUPPORTED.
 * Errors: NULL, SHAPE (even kernel, K != Cin * kh * kw, ldy < H * W, sizes < 1), DEVICE, UNSUPPORTED.
 */
grim_status grim_bcr_conv2d(const grim_bcr_matrix *A, const void *F_dev, int32_t Cin, int32_t H, int32_t W,
                            int32_t kh, int32_t kw, float *Y_dev, int64_t ldy, void *hip_stream);

/*
 * grim_bcr_conv2d_act -- the same convolution with the rest of a CONV layer in its epilogue (Section 6.1:
 * the evaluated networks are chains of CONV + bias + rectifier layers, run in fp16 on the GPU):
 *     out[m][n] = round_to(out_dt, act(Y[m][n] + bias[m])),   act = max(., 0) when relu != 0, else identity
 *   bias_dev  M fp32, or NULL (no bias)
 *   out_dev   M x (H * W) of element type out_dt (fp32, fp16 or bf16; round to nearest even), leading
 *             dimension ldo >= H * W, overwritten.  In fp16 / bf16 it is the next layer's feature map
 *             (M channels of H x W) as it stands.  Must not overlap F_dev.
 * Sums are accumulated in fp32 exactly as in grim_bcr_conv2d; with out_dt = GRIM_F32, no bias and no
 * rectifier the two calls write the same bits.  Conditions and errors as grim_bcr_conv2d; an unknown
 * out_dt is GRIM_ERR_DTYPE.
 */
grim_status grim_bcr_conv2d_act(const grim_bcr_matrix *A, const void *F_dev, int32_t Cin, int32_t H, int32_t W,
                                int32_t kh, int32_t kw, const float *bias_dev, int32_t relu, void *out_dev,
                                grim_dtype out_dt, int64_t ldo, void *hip_stream);

/*
 * Convolution plan: a packed filter matrix bound to one layer geometry (Section 3.1: CONV as the filter matrix times
 * the im2col matrix; Section 4.5: rows of that matrix whose weights are pruned are skipped).  For every row of the
 * im2col matrix the matrix keeps, the plan holds where in a feature map that row starts (input channel, kernel row
 * and column folded into one offset) and which kernel tap it is, so that the kernel does not split row numbers while
 * it runs; it also carries a stride and serves a batch of images in one launch.
 *   grim_bcr_conv_plan_create   A: packed M x (Cin * kh * kw) on the current device (must outlive the plan);
 *                               kh, kw odd, padding kh / 2, kw / 2; stride 1 or 2 in both directions; the output
 *                               map is Ho x Wo = ceil(H / stride) x ceil(W / stride).  Allocates the plan's words
 *                               (4 bytes per kept im2col row, padded) on the device.  Errors: NULL, SHAPE, DEVICE,
 *                               ALLOC, UNSUPPORTED (as grim_bcr_conv2d).
 *   grim_bcr_conv2d_plan        F_dev: batch images [Cin][H][W] of A's element type, image b at F_dev +
 *                               b * f_image_stride elements; out_dev: batch outputs [M][ldo] (ldo >= Ho * Wo) of
 *                               element type out_dt, image b at out_dev + b * out_image_stride elements, overwritten
 *                               (entries n < Ho * Wo of each row); bias_dev (M fp32 or NULL), relu and the rounding as
 *                               grim_bcr_conv2d_act.  With batch = 1 the image strides are ignored.  Sums in fp32 in
 *                               the same order as grim_bcr_conv2d: with stride 1 the two write the same bits.  Stride 2
 *                               computes on the input grid and stores the even positions (every second row is skipped
 *                               when W is a multiple of 8).  Enqueues one launch on hip_stream, allocates nothing.
 *                               Errors: NULL, SHAPE (batch < 1, ldo or an image stride too small), DTYPE, DEVICE,
 *                               UNSUPPORTED.
 *   grim_bcr_conv_plan_free     frees the plan (not the matrix).
 */
/* grim_bcr_conv2d_kernel_name -- which kernel grim_bcr_conv2d / _act (batch 1, stride 1) or grim_bcr_conv2d_plan runs for
 * this layer with densely stored, 16-byte aligned operands ("bcr_conv_wide": the wide-tile kernel, for stride-1 layers of
 * at least 8 row strips with at least one round of 256 workgroups' worth of positions whose H * W is a multiple of 8; "bcr_conv_gather";
 * "none": refused).  A static string; launches nothing. */
const char *grim_bcr_conv2d_kernel_name(const grim_bcr_matrix *A, int32_t Cin, int32_t H, int32_t W, int32_t kh, int32_t kw,
                                        int32_t batch, int32_t stride);
typedef struct grim_bcr_conv_plan grim_bcr_conv_plan;
grim_status grim_bcr_conv_plan_create(const grim_bcr_matrix *A, int32_t Cin, int32_t H, int32_t W, int32_t kh, int32_t kw,
                                      int32_t stride, grim_bcr_conv_plan **out);
void grim_bcr_conv_plan_free(grim_bcr_conv_plan *plan);
grim_status grim_bcr_conv2d_plan(const grim_bcr_conv_plan *plan, const void *F_dev, int32_t batch, int64_t f_image_stride,
                                 const float *bias_dev, int32_t relu, void *out_dev, grim_dtype out_dt, int64_t ldo,
                                 int64_t out_image_stride, void *hip_stream);

/*
 * LSTM cell around the gate product (Section 3.1: an RNN layer's gate matrices are one matrix-vector
 * product per time step).  With the gate matrix [W_ih | W_hh] of 4H rows packed as one BCR matrix
 * and the step's input vector [x; h], grim_bcr_spmv delivers the gate pre-activations, rows [0, H)
 * input gate, [H, 2H) forget gate, [2H, 3H) cell candidate, [3H, 4H) output gate (the order is this
 * library's convention; the paper does not fix one).  grim_lstm_cell is the elementwise rest:
 *     i, f, o = sigmoid(gate + bias), g = tanh(gate + bias), c <- f * c + i * g, h = o * tanh(c)
 * in fp32; sigmoid(v) = 1 / (1 + 2^(-v log2 e)) and tanh(v) = 1 - 2 / (1 + 2^(2 v log2 e)) on the GPU's
 * exponential and reciprocal instructions (1 ulp each): absolute error below 2e-7, saturating to 0 / 1 / -1
 * for large arguments, NaN in, NaN out.  The cell kernels, the one-launch steps and the sequence entry points
 * share this arithmetic and agree bit for bit.  (The GRU cell below uses the same two functions.)
 *   gates_dev   4H x batch fp32, leading dimension ldg >= batch
 *   bias_dev    4H fp32 or NULL
 *   c_dev       H x batch fp32 (ldc), read and overwritten
 *   h_dev       H x batch of element type dt (ldh), written; typically the h part of the next step's
 *               input vector.  May be NULL.
 *   h32_dev     optional fp32 copy of h (ldh32); NULL to skip
 * grim_bcr_lstm_step = grim_bcr_spmv(A, xh_dev, ...) (more than 8 columns: grim_bcr_spmm) into
 * gates_dev, then grim_lstm_cell; A must have 4H rows.  Both only enqueue work on hip_stream.
 * With fp16 / bf16, every block of A keeping the same number of rows and of columns, H a multiple of BR, h_dev
 * outside the vectors xh_dev (write the new h into the NEXT step's input vectors) and batch x H / BR workgroups no
 * more than the GPU's compute units (batch <= 8 for H = 1024 in 32-row strips), the step is ONE launch: each
 * workgroup computes the four gate rows of BR hidden units for one column and applies the cell before it stores
 * anything (gates_dev still receives the pre-activations).  Otherwise two launches.
 * Errors: NULL, SHAPE (batch < 1, H < 1, leading dimension too small, A->M != 4H), DTYPE, DEVICE,
 * UNSUPPORTED.
 */
/* grim_bcr_rnn_step_launches -- how many kernels a recurrent step enqueues (for reports and tests; launches nothing):
 * grim_bcr_lstm_step of A (Ah = NULL) or grim_bcr_gru_step of (A, Ah) at this batch, for operands with the usual
 * alignment and a new state that does not overlap the step's inputs.  1 = the gate product(s) with the cell in the
 * epilogue; 2 = product(s) in one launch, then the cell; 3 = a launch per product, then the cell; 0 = the step would
 * be refused. */
int32_t grim_bcr_rnn_step_launches(const grim_bcr_matrix *A, const grim_bcr_matrix *Ah, int32_t batch);

grim_status grim_lstm_cell(const float *gates_dev, int64_t ldg, const float *bias_dev, float *c_dev, int64_t ldc,
                           void *h_dev, grim_dtype dt, int64_t ldh, float *h32_dev, int64_t ldh32,
                           int64_t H, int32_t batch, void *hip_stream);
grim_status grim_bcr_lstm_step(const grim_bcr_matrix *A, const void *xh_dev, int32_t batch, int64_t ldx,
                               float *gates_dev, int64_t ldg, const float *bias_dev, float *c_dev, int64_t ldc,
                               void *h_dev, int64_t ldh, float *h32_dev, int64_t ldh32, void *hip_stream);

/*
 * GRU cell around the gate products (Section 6.1: the evaluated RNN is a two-layer GRU, timed in Section 6.3; its layers are the
 * matrix-vector products of Section 3.1).  Two BCR matrices of 3H rows each, W_i (3H x I) and
 * W_h (3H x H), gate rows stacked reset, update, candidate; gi = W_i x and gh = W_h h come from
 * grim_bcr_spmv / grim_bcr_spmm, grim_gru_cell is the elementwise rest (the standard GRU with the
 * reset gate applied to the hidden-side candidate product; the paper does not restate the cell):
 *     r = sigmoid(gi_r + bi_r + gh_r + bh_r)      z = sigmoid(gi_z + bi_z + gh_z + bh_z)
 *     n = tanh(gi_n + bi_n + r * (gh_n + bh_n))   h <- (1 - z) * n + z * h
 *   gi_dev, gh_dev   3H x batch fp32 (ldgi, ldgh >= batch)
 *   bias_i_dev, bias_h_dev   3H fp32 each, or NULL
 *   h32_dev   H x batch fp32 (ldh32): the state, read and overwritten
 *   h_dev     optional copy of the new state in element type dt (ldh): what the next step's
 *             hidden-side product reads.  May be NULL.
 * grim_bcr_gru_step = the two products (x_dev: I x batch, hin_dev: H x batch, both of the matrices'
 * element type; any batch >= 1: up to 8 columns run on the SpMV kernels, more on the SpMM kernels;
 * with equal leading dimensions on both sides one launch computes both products -- on the SpMV
 * kernels for W_i and W_h of one shape and block size, on the row-gathering SpMM kernel for 4 to 60
 * columns in multiples of 4)
 * into gi_dev and gh_dev, then grim_gru_cell writing hout_dev (may be hin_dev itself: the cell runs
 * after both products).  With fp16 / bf16 matrices of one shape, block size and kept counts, H a multiple of BR,
 * hout_dev overlapping neither x_dev nor hin_dev, and batch x H / BR workgroups no more than the GPU's compute
 * units, the step is ONE launch (products with the cell in their epilogue, a set of workgroups per column;
 * gi_dev / gh_dev still receive the products).  Both only enqueue work on hip_stream.  Errors: NULL, SHAPE (rows not 3H on
 * both, Ah->K != H, batch < 1, leading dimension too small), DTYPE (element types differ), DEVICE,
 * UNSUPPORTED (as the products).
 */
grim_status grim_gru_cell(const float *gi_dev, int64_t ldgi, const float *gh_dev, int64_t ldgh,
                          const float *bias_i_dev, const float *bias_h_dev, float *h32_dev, int64_t ldh32,
                          void *h_dev, grim_dtype dt, int64_t ldh, int64_t H, int32_t batch, void *hip_stream);
grim_status grim_bcr_gru_step(const grim_bcr_matrix *Ai, const grim_bcr_matrix *Ah, const void *x_dev, int64_t ldx,
                              const void *hin_dev, int64_t ldhin, int32_t batch, float *gi_dev, int64_t ldgi,
                              float *gh_dev, int64_t ldgh, const float *bias_i_dev, const float *bias_h_dev,
                              float *h32_dev, int64_t ldh32, void *hout_dev, int64_t ldhout, void *hip_stream);

/*
 * A recurrent layer over a whole sequence in ONE launch (Section 3.1: one matrix-vector product per time step;
 * Section 6.3 times the recurrent network step by step).  The weights are read once and stay in registers for all T
 * steps; workgroups (one per BR hidden units, all resident at once) hand the new hidden state to each other through
 * a small exchange buffer that belongs to the matrix (A, or Ah for the GRU), allocated by the first such call.
 *   grim_bcr_lstm_sequence   A: the gate matrix [W_ih | W_hh], 4H x (I + H), as for grim_bcr_lstm_step
 *   grim_bcr_gru_sequence    Ai: 3H x I, Ah: 3H x H, as for grim_bcr_gru_step
 *   xs_dev     T x I inputs in the matrices' element type, row t at xs_dev + t * ldxs elements (ldxs >= I)
 *   bias*_dev  as for the step calls, or NULL
 *   h0_dev     H elements (element type of the matrices): the hidden state the first step's product reads
 *   c_dev      LSTM: H fp32, cell state, read before the first step and overwritten with the last step's
 *   h32_dev    GRU: H fp32, hidden state in fp32 (the z * h term reads it), read and overwritten likewise
 *   hs_dev     T x H outputs h_1 .. h_T in the matrices' element type (ldhs >= H), overwritten; hs32_dev: the same in
 *              fp32 (ldhs32 >= H), or NULL.  Step t + 1 reads h_t rounded to the element type, as a chain of step
 *              calls does, and computes the same values as that chain.
 *   status_dev one int32 on the device, overwritten: 0 = done, 1 = a workgroup gave up waiting for another
 *              workgroup's state (the GPU was too busy to hold all workgroups at once for longer than the limit); the
 *              outputs are then undefined.  The caller reads it after synchronising with hip_stream.
 *   max_polls  limit of unsuccessful reads of an exchange word before a workgroup gives up; 0 = default (2^21,
 *              seconds).  Every workgroup leaves the kernel either way.
 * The *_batch forms run `batch` independent sequences (1 .. 32) in the same launch, spread over further sets of
 * H / BR workgroups while the GPU has compute units for them and several per workgroup beyond that:
 * row t * batch + b of xs_dev / hs_dev / hs32_dev belongs to step t of sequence b; h0_dev is batch x H elements,
 * c_dev / h32_dev batch x H fp32, sequence b at offset b * H.  Every sequence gets the bits a call of its own
 * with batch 1 would give.  More than 32, or a workgroup's vectors not fitting its local memory
 * (sequences per workgroup x (I + H) x 2 bytes plus tables within 160 KB): GRIM_ERR_UNSUPPORTED;
 * grim_bcr_rnn_sequence_batch_supported tells in advance.  The calls without _batch are batch = 1.
 * The exchange buffer holds 2 x 32 x H words of 8 bytes.
 * Requirements: fp16 / bf16, blocks of at most 32 x 32 all keeping the same (rows, columns)
 * out of {4, 8, 16} x {4, 8, 12, 16} (not 16 x 16), at most 64 column blocks per matrix, H a multiple of BR,
 * H <= 8192 and H / BR workgroups <= the GPU's compute units; otherwise GRIM_ERR_UNSUPPORTED (loop over the step
 * call instead); grim_bcr_rnn_sequence_supported(A, Ah or NULL) tells in advance (1 / 0).
 * Two sequence calls on the same matrix must not overlap in time (they share the exchange buffer): enqueue them
 * on one stream.  Only enqueues work on hip_stream (two launches: clearing the exchange words, the sequence).
 * Errors: NULL, SHAPE (T < 1, batch < 1, rows not 4H / 3H, leading dimension too small), DTYPE, DEVICE, ALLOC,
 * UNSUPPORTED.
 */
int32_t grim_bcr_rnn_sequence_supported(const grim_bcr_matrix *A, const grim_bcr_matrix *Ah);
int32_t grim_bcr_rnn_sequence_batch_supported(const grim_bcr_matrix *A, const grim_bcr_matrix *Ah, int32_t batch);
grim_status grim_bcr_lstm_sequence(const grim_bcr_matrix *A, const void *xs_dev, int64_t ldxs, int32_t T,
                                   const float *bias_dev, const void *h0_dev, float *c_dev, void *hs_dev, int64_t ldhs,
                                   float *hs32_dev, int64_t ldhs32, int32_t *status_dev, uint32_t max_polls,
                                   void *hip_stream);
grim_status grim_bcr_gru_sequence(const grim_bcr_matrix *Ai, const grim_bcr_matrix *Ah, const void *xs_dev, int64_t ldxs,
                                  int32_t T, const float *bias_i_dev, const float *bias_h_dev, const void *h0_dev,
                                  float *h32_dev, void *hs_dev, int64_t ldhs, float *hs32_dev, int64_t ldhs32,
                                  int32_t *status_dev, uint32_t max_polls, void *hip_stream);
grim_status grim_bcr_lstm_sequence_batch(const grim_bcr_matrix *A, const void *xs_dev, int64_t ldxs, int32_t T, int32_t batch,
                                         const float *bias_dev, const void *h0_dev, float *c_dev, void *hs_dev, int64_t ldhs,
                                         float *hs32_dev, int64_t ldhs32, int32_t *status_dev, uint32_t max_polls,
                                         void *hip_stream);
grim_status grim_bcr_gru_sequence_batch(const grim_bcr_matrix *Ai, const grim_bcr_matrix *Ah, const void *xs_dev, int64_t ldxs,
                                        int32_t T, int32_t batch, const float *bias_i_dev, const float *bias_h_dev,
                                        const void *h0_dev, float *h32_dev, void *hs_dev, int64_t ldhs, float *hs32_dev,
                                        int64_t ldhs32, int32_t *status_dev, uint32_t max_polls, void *hip_stream);

/*
 * grim_bcr_lstm_sequence_noalloc -- grim_bcr_lstm_sequence for callers that cannot allocate device memory (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, same kernels,
 * same results, but the exchange words live in a static device array of the library (2 x 8192 words of 8 bytes
 * = 128 KB per GPU, held until the process ends) instead of a buffer allocated with the matrix.  The call
 * allocates and frees nothing, on the device or through any library.  H > 8192 is GRIM_ERR_UNSUPPORTED.  All such
 * calls on one GPU share the array (whatever the matrix): calls that overlap in time on one GPU race -- enqueue them
 * on one stream.  The words are cleared by a small kernel at the start of every call, so the call can be captured.
 * Errors as grim_bcr_lstm_sequence (no ALLOC).
 */
grim_status grim_bcr_lstm_sequence_noalloc(const grim_bcr_matrix *A, const void *xs_dev, int64_t ldxs, int32_t T,
                                           const float *bias_dev, const void *h0_dev, float *c_dev, void *hs_dev,
                                           int64_t ldhs, float *hs32_dev, int64_t ldhs32, int32_t *status_dev,
                                           uint32_t max_polls, void *hip_stream);


/*
 * BCRC export (Section 4.3, "Compact Model Storage"): the paper's six-array, row-level form of the
 * same pruned matrix.  Rows of the whole matrix are reordered so that rows with the same set of
 * kept (global) columns are adjacent -- groups in order of the first original row that shows the
 * pattern, rows inside a group in ascending original order -- and the column indices of a group are
 * stored once:
 *   reorder[M]            original row id of reordered row p            (the paper's `reorder`)
 *   row_offset[M+1]       start of reordered row p in weights           (`row offset`)
 *   occurrence[G+1]       first reordered row of each group             (`occurrence`)
 *   column_stride[G+1]    start of each group's list in compact_column  (`column stride`)
 *   compact_column[...]   global column indices of each group, ascending (`compact column`)
 *   weights[nnz]          reordered rows, each its kept weights in column order (`weights`)
 * Rows that keep nothing form one group with an empty column list.  Host-only (works on matrices
 * packed with host_only); the arrays are owned by the grim_bcrc object.
 */
typedef struct grim_bcrc grim_bcrc;
typedef struct grim_bcrc_view {
    int64_t M, K, ngroups, nnz, ncols;   /* ncols = length of compact_column */
    int32_t dtype;
    const int32_t *reorder;
    const int64_t *row_offset;
    const int32_t *occurrence;
    const int64_t *column_stride;
    const int32_t *compact_column;
    const void *weights;
} grim_bcrc_view;
grim_status grim_bcr_export_bcrc(const grim_bcr_matrix *A, grim_bcrc **out);   /* NULL, ALLOC */
grim_status grim_bcrc_arrays(const grim_bcrc *B, grim_bcrc_view *v);
void grim_bcrc_free(grim_bcrc *B);

/* grim_bcr_free -- release a matrix and its device memory.  NULL is a no-op. */
void grim_bcr_free(grim_bcr_matrix *A);

/* grim_status_str -- static, human-readable name of a status code. */
const char *grim_status_str(grim_status s);

#ifdef __cplusplus
}
#endif
#endif /* GRIM_BCR_H */

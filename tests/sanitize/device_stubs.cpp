// Stand-ins for the kernel launchers, so that the host side of the library (validation, compaction, the
// derived layouts, their decoders, the BCRC export) links without any device code and can run under the
// address and undefined-behaviour sanitizers on a machine without a GPU.  Every launcher reports that
// there is no device; nothing here computes anything.
#include "bcr_matrix.hpp"

namespace grim {
grim_status launch_spmm_fma(const grim_bcr_matrix *, const void *, int64_t, int64_t, float *, int64_t, hipStream_t) { return GRIM_ERR_DEVICE; }
grim_status launch_spmm_mma(const grim_bcr_matrix *, const void *, int64_t, int64_t, float *, int64_t, int32_t, int32_t, hipStream_t) { return GRIM_ERR_DEVICE; }
bool mma_supported(const grim_bcr_matrix *) { return false; }
grim_status launch_spmm_wide(const grim_bcr_matrix *, const void *, int64_t, int64_t, float *, int64_t, int32_t, hipStream_t) { return GRIM_ERR_DEVICE; }
grim_status launch_spmm_wide_with_rest(const grim_bcr_matrix *, const void *, int64_t, int64_t, float *, int64_t, int32_t, int64_t, hipStream_t) { return GRIM_ERR_DEVICE; }
bool wide_applies(const grim_bcr_matrix *, const void *, int64_t, int64_t, const float *, int64_t, int32_t) { return false; }
double wide_plan(const grim_bcr_matrix *, const void *, int64_t, int64_t, const float *, int64_t, double (*)(const grim_bcr_matrix *, int64_t), int *, int64_t *) { return -1.0; }
grim_status launch_spmm_gather(const grim_bcr_matrix *, const void *, int64_t, int64_t, float *, int64_t, hipStream_t, const grim_bcr_matrix *, const void *, float *) { return GRIM_ERR_DEVICE; }
bool gather_pair_applies(const grim_bcr_matrix *, const void *, const grim_bcr_matrix *, const void *, int64_t, int64_t) { return false; }
bool gather_applies(const grim_bcr_matrix *, const void *, int64_t, int64_t) { return false; }
bool gather_wave_per_strip(const grim_bcr_matrix *, int64_t, int64_t) { return false; }
grim_status launch_conv_gather(const grim_bcr_matrix *, const void *, int32_t, int32_t, int32_t, int32_t, int32_t, const float *, int32_t, void *, int32_t, int64_t, hipStream_t, int32_t, int32_t, int64_t, int64_t, const uint32_t *, int32_t, int64_t, int64_t) { return GRIM_ERR_DEVICE; }
uint32_t conv_plan_word(uint32_t, int32_t, int32_t, int32_t, int32_t) { return 0; }
bool conv_wide_applies(const grim_bcr_matrix *, const void *, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, int64_t, const void *, int32_t, int64_t, int64_t) { return false; }
grim_status launch_conv_wide(const grim_bcr_matrix *, const void *, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, int64_t, const float *, int32_t, void *, int32_t, int64_t, int64_t, hipStream_t) { return GRIM_ERR_UNSUPPORTED; }
double gather_cost(const grim_bcr_matrix *, int64_t) { return 0.0; }
double mma_best_shape(const grim_bcr_matrix *, int64_t, int32_t, int32_t, int *, int *) { return -1.0; }
int64_t mma_whole_rounds(const grim_bcr_matrix *, int64_t N, bool, int *, int *) { return N; }
grim_status launch_spmv(const GemvDesc *, const GemvDesc &, const GemvDesc *, int32_t, int64_t, int64_t, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, const void *, int64_t, int32_t, int64_t, float *, int64_t, int64_t, hipStream_t) { return GRIM_ERR_DEVICE; }
bool spmv_cell_applies(int, int64_t, int64_t, int32_t, int32_t, int32_t, int32_t, int32_t, int64_t) { return false; }
grim_status launch_spmv_cell(int, const GemvDesc &, const GemvDesc *, int64_t, int64_t, int32_t, int32_t, int32_t, int32_t, int32_t, const void *, int64_t, int32_t, int64_t, float *, int64_t, int64_t, const RnnCell &, hipStream_t) { return GRIM_ERR_DEVICE; }
grim_status rnn_seq_static_exchange(void **) { return GRIM_ERR_DEVICE; }
bool spmv_cell_batch_ok(int64_t, int32_t, int32_t) { return false; }
bool spmv_exact_applies(int32_t, int32_t, int32_t, int64_t) { return false; }
bool spmv_column_sets_ok(int64_t, int64_t, int32_t) { return false; }
bool rnn_seq_applies(int, int32_t, int32_t, int32_t, int32_t, int32_t, int64_t, int64_t, int64_t, int64_t, int32_t) { return false; }
grim_status launch_rnn_seq(int, const GemvDesc &, const GemvDesc *, const int32_t *, const int32_t *, int32_t, int32_t, int32_t, int32_t, int32_t, int64_t, int64_t, int64_t, int64_t, int32_t, int32_t, const void *, int64_t, const void *, const float *, const float *, float *, void *, int64_t, float *, int64_t, void *, int32_t *, uint32_t, hipStream_t) { return GRIM_ERR_DEVICE; }
grim_status launch_lstm_cell(const float *, int64_t, const float *, float *, int64_t, void *, int32_t, int64_t, float *, int64_t, int64_t, int32_t, hipStream_t) { return GRIM_ERR_DEVICE; }
grim_status launch_gru_cell(const float *, int64_t, const float *, int64_t, const float *, const float *, float *, int64_t, void *, int32_t, int64_t, int64_t, int32_t, hipStream_t) { return GRIM_ERR_DEVICE; }
}  // namespace grim

// the HIP runtime calls the host side makes (allocation and upload of a packed matrix): no device here
extern "C" {
hipError_t hipGetDeviceCount(int *n) { if (n) *n = 0; return hipErrorNoDevice; }
hipError_t hipGetDevice(int *d) { if (d) *d = -1; return hipErrorNoDevice; }
hipError_t hipGetLastError(void) { return hipSuccess; }
hipError_t hipMalloc(void **p, size_t) { if (p) *p = nullptr; return hipErrorNoDevice; }
hipError_t hipFree(void *) { return hipErrorNoDevice; }
hipError_t hipMemset(void *, int, size_t) { return hipErrorNoDevice; }
hipError_t hipMemcpy(void *, const void *, size_t, hipMemcpyKind) { return hipErrorNoDevice; }
}

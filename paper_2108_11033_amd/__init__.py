"""BCR (Block-based Column-Row) sparse SpMM / SpMV for AMD MI355X.

Thin ctypes binding of libgrim_bcr.so (see include/grim_bcr.h).  All arithmetic
runs in the library's HIP kernels; this package only marshals arguments.
"""
from .binding import (  # noqa: F401
    BcrMatrix, BcrGroup, GrimError, lib_path, load_library, pack, conv2d, conv2d_act, ConvPlan, conv2d_plan, conv2d_kernel_name, export_bcrc, lstm_cell, lstm_step, rnn_step_launches, rnn_sequence_supported, lstm_sequence, lstm_sequence_noalloc, gru_sequence, lstm_sequence_batch, gru_sequence_batch, gru_cell, gru_step, spmm, spmm_kernel_name, spmv, spmv_batched,
    F32, F16, BF16, STATUS_NAMES,
)

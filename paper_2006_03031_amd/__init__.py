"""MI355X-native dynamic-shape dense / batch_matmul / LSTM-cell path.

Thin ctypes binding over the C ABI declared in ``include/nimble.h``; every step
of the path runs in the HIP library.  PyTorch is used by callers only for
device memory and streams.
"""
from .binding import (  # noqa: F401
    EPI_BIAS, EPI_BIAS_GELU_ERF, EPI_NONE, BF16, F32, VAR_AUTO, NimbleError, Plan,
    batch_matmul_plan, batch_matmul_shape, dense_plan, dense_table_set, dense_shape, last_error, library_path, load,
    lstm_plan, lstm_shape, lstm_pre_shape, nimble_batch_matmul_dyn, nimble_dense_dyn, nimble_dense_variant_dyn, nimble_dense_noalloc_dyn, NOALLOC_SCRATCH_BYTES,
    nimble_dense_shape,
    nimble_attention_dyn, nimble_lstm_gates_dyn, nimble_lstm_gates_pre_dyn, nimble_softmax_rows_dyn, residue_split, storage_alignment, storage_bytes,
    lstm_seq_shape, lstm_seq_supported, lstm_seq_preferred, lstm_seq_workspace_bytes, nimble_lstm_seq_pre_dyn, nimble_lstm_seq_status,
    variant_name, exported_symbols, nimble_probe_mfma_bf16, nimble_probe_hbm_read,
)

"""SJD++ (speculative Jacobi decoding with token reuse) on one MI355X: thin Python binding of libsjd.so.

Only argument marshalling lives here; every step of the decoding path runs in the HIP library.
"""
from .binding import (SjdError, Decoder, lib, library_path, op_gemm, op_gemm_static, op_window_attention, op_sampling_rows,  # noqa: F401
                      op_philox, KERNELS_REFERENCE, NO_GRAPH, KERNELS_ROWGROUPS, ATTENTION_CHUNKED, KERNELS_TILES, NO_L2_WARM, TILES_256_ROWS, NO_ROW_SPLIT, NO_MIXED_WIDTH, NO_K_ROTATION, KEEP_LOGITS, NO_HEAD_FUSION, F32, BF16,
                      OK, EINVAL, ENOMEM, ESTATE, EDEVICE, ECAPACITY)

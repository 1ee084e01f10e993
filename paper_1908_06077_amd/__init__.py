"""NUQSGD gradient-compression hot path for AMD MI355X: thin binding over libnuq.so.

Every function here only marshals arguments (torch tensors -> device pointers, the current
HIP stream) into the C ABI declared in include/nuq.h; all steps of the path run in the HIP
kernels.  There is no CPU fallback: importing the package fails if the library is missing.
"""
from .binding import (  # noqa: F401
    NuqError, Message,
    FLAG_CAPACITY, FLAG_NONFINITE, FLAG_MALFORMED, SYNC_BLOCK, MAX_BUCKET, MAX_S, MAX_WORKERS,
    nuq_num_buckets, nuq_num_sync, nuq_huffman_num_sync, nuq_max_words, nuq_encode_workspace_bytes, nuq_workspace_bytes,
    nuq_bucket_norms, nuq_quantize, nuq_encode, nuq_quantize_encode, nuq_quantize_encode_batch, nuq_decode_accumulate,
    nuq_quantize_encode_static, STATIC_WORKSPACE_BYTES,
    nuq_bucket_norms_linf, nuq_quantize_table, nuq_quantize_encode_table_batch, nuq_decode_accumulate_table,
    NORM_L2, NORM_LINF,
    nuq_level_histogram, nuq_huffman_lengths, nuq_huffman_max_words, nuq_encode_huffman_workspace_bytes,
    nuq_encode_huffman, nuq_encode_huffman_batch_workspace_bytes, nuq_quantize_encode_huffman_batch, nuq_decode_huffman, nuq_decode_huffman_batch, nuq_average_levels, nuq_decode_accumulate_huffman,
    nuq_fixed_words, nuq_pack_fixed, nuq_quantize_pack_fixed_batch, nuq_unpack_accumulate_fixed,
    nuq_quantize_pack_fixed_table_batch, nuq_unpack_accumulate_fixed_table,
    nuq_momentum_step, nuq_decode_momentum_step, nuq_moments_accumulate, nuq_normalized_variance, VARIANCE_WORKSPACE_BYTES,
    nuq_last_error_flags, library_path, exported_symbols,
    nuq_timing_begin, nuq_timing_collect, T_NORMS, T_QUANTIZE, T_ENCODE, T_QUANTIZE_ENCODE, T_DECODE,
)

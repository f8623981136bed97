"""MI355X-native EasyQuant quantization path: thin Python binding over libeasyquant.so.

The library (hand-written HIP for gfx950 behind a C ABI, see include/easyquant.h) does all
the work; this package only marshals arguments.  PyTorch provides device memory and streams.
There is no CPU fallback: importing `binding` fails loudly if the library is not built.
"""
from .binding import (  # noqa: F401
    EQ_ASYMMETRIC, EQ_BF16, EQ_F16, EQ_SELECT_BEST, EQ_SELECT_LAST, EQ_STAT_GROUP, EQ_STAT_MATRIX, EQ_STAT_ROW,
    EQ_SYMMETRIC, EQ_S_NONFINITE, EQ_S_OUTLIER_OVERFLOW, EasyQuantError, Params, QMatrix, eq_code_words_per_row,
    eq_dequant_matvec, eq_dequantize, eq_outlier_capacity_bound, eq_profile_enable, eq_profile_read, eq_quantize_batch, eq_quantize_matrix, eq_quantize_matrix_noalloc, EQ_STATIC_SCRATCH_BYTES, eq_strerror, eq_workspace_bytes,
    alloc_outputs, lib, lib_path,
    OVR_CHANNEL_KERNEL, OVR_FORCE_GENERAL, OVR_MATVEC_ARITHMETIC, OVR_MATVEC_LOOKUP, OVR_RTN_THREADS, OVR_UNITS_PER_ITEM, OVR_SORTED_ROWS, OVR_SORT_CHUNK_ROWS, OVR_CLASS_STREAMS, OVR_COUNT,
    override, plan_items, plan_sort_segments,
    set_override,
)

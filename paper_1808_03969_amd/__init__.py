"""MI355X-native search path of the reconfigurable inverted index (Rii).

Thin Python binding over the C-ABI library ``librii_hip.so`` (see ``include/rii.h``): the
functions here have the library's names and only marshal arguments.  Every step of the path
runs in the library's HIP kernels; PyTorch supplies device memory and streams.
"""
from .binding import (  # noqa: F401
    RiiError, Index, load_library, library_path,
    rii_train_codebooks, rii_encode, rii_build_lut, rii_coarse_assign, rii_adc_scan_linear,
    rii_adc_scan_subset, rii_adc_scan_ivf, rii_topk, rii_query, rii_encode_device, rii_assign,
    rii_index_set_scan_events, rii_rotate, rii_check_target_ids, rii_query_noalloc,
)

"""tq: dictionary-coded int8 weights kept compressed in HBM, fused decode + dequantize + GEMV on MI355X.

Thin ctypes binding over libtq.so (C ABI in include/tq.h).  Argument marshalling only: every step of the
hot path runs in the library's HIP kernels.  Importing this package never falls back to a CPU path; if the
library has not been built, loading it raises.
"""
from .binding import (  # noqa: F401
    TQ_MAX_BATCH,
    TQ_MAX_ENTRIES_DEVICE,
    TQ_MAX_LMAX,
    TQ_DEFAULT_SEG_COLS,
    TqError,
    TqInfo,
    Matrix,
    lib_path,
    load,
    tq_encode,
    tq_encode_quantized,
    tq_validate_blob,
    tq_create_from_encoded,
    tq_matvec,
    tq_matvec_multi,
    tq_set_ring_min_bands_per_cu,
    MultiCall,
    tq_decompress,
    tq_decompress_multi,
    tq_get_info,
    tq_destroy,
    tq_last_error_string,
    TqListingInfo,
    Listing,
    tq_listing_build_table,
    tq_listing_compress,
    tq_encode_gate_up,
    tq_matvec_gate_up,
    tq_matvec_gate_up_multi,
    TQ_STEP_GATE_UP,
    TQ_STEP_DECOMPRESS,
    Step,
    tq_step_create,
    tq_step_launch,
    tq_step_get_info,
    tq_step_destroy,
)

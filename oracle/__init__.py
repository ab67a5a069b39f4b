"""CPU oracle of the output-equivalence check.  TEST INFRASTRUCTURE ONLY.

Imported by tests/, by the smoke check and by the benchmark's CPU-baseline leg.
The product package never imports it.
"""
from .oracle import (  # noqa: F401
    RECORD_DTYPE,
    MISMATCH_DTYPE,
    DTYPE_CODES,
    ELEM_SIZE,
    build,
    check_segment,
    report_segment,
    ulp_histogram_segment,
    ULP_BINS,
    check_dense,
    check_ragged,
    check_dense_chunked,
    check_segment_mapped,
    check_segment_nd,
    gather_nd,
    gather_rows,
    combine_records,
    host_cores,
    decode_f8,
    decode_f16,
    decode_bf16,
)

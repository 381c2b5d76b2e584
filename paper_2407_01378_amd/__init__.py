"""MI355X-native chunked-RHT stochastic gradient quantization (THC case study).

The work is done by hand-written gfx950 HIP kernels behind a C ABI
(include/thc.h, built into libthc.so by paper_2407_01378_amd.build); this
package is the thin ctypes binding with the same names.
"""
from .binding import (  # noqa: F401
    THC_BF16,
    THC_F32,
    THC_OK,
    ThcError,
    exported_names,
    lib,
    rht_forward,
    rht_inverse,
    status_string,
    thc_aggregate,
    thc_aggregate_decode,
    thc_aggregate_decode_is_fused,
    thc_encode_all,
    thc_encode_all_timed_out,
    thc_encode_all_workspace_bytes,
    thc_set_spin_limit,
    thc_chunk_absmax,
    thc_decode,
    thc_encode,
    thc_num_chunks,
    thc_payload_bytes,
    thc_rounding_bits,
    thc_sat_aggregate,
    thc_sat_aggregate_decode,
    thc_sat_aggregate_decode_is_fused,
    thc_sat_decode,
    thc_sat_encode,
    thc_sat_encode_all,
    thc_sat_max,
    thc_scale_reduce,
    thc_sum_bytes,
    thc_version,
)

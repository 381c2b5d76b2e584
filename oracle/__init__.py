"""CPU oracle for the chunked-RHT stochastic quantization path (THC case study).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library and its
Python binding) may import, call or link anything from this package; only the
tests, the smoke check and the benchmark's cpu_baseline leg do.  The oracle is
plain NumPy, written from the paper's description (THC background and
"Our proposed improvements": partial rotation, per-chunk range, stochastic
rounding to q-bit integers, integer summation with b >= q bits) and shares no
code, tables or helpers with the GPU implementation.

Parity status: every function is pinned by closed forms, invariants or brute
force in the CPU test-suite.  Absolute agreement with the paper authors' own
prototype is "parity unpinned": the paper prints no worked numeric example of
its rotation or quantizer, so only the mathematics fixes the values.
"""

from .philox import philox4x32_10, philox4x32_10_scalar  # noqa: F401
from .thc import (  # noqa: F401
    RBITS,
    TAG_ROUND,
    TAG_SIGN,
    aggregate,
    chunk_absmax,
    decode,
    fwht,
    num_chunks,
    pack,
    payload_bytes,
    pipeline,
    quantize,
    rht_forward,
    rht_inverse,
    rounding_fields,
    scale_reduce,
    sign_bits,
    sum_dtype,
    unpack,
)

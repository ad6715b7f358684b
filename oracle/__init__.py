"""CPU oracle for the Distributed Lion optimizer sweep -- TEST INFRASTRUCTURE.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It shares no code with the HIP library and the product path never
calls it.  See ``dlion_oracle.c`` for the arithmetic (Algorithm 1; Section 3.2)
and ``dlion_oracle.py`` for the numpy-facing wrapper.
"""
from .dlion_oracle import (  # noqa: F401
    AVG,
    Oracle,
    SOURCE,
    VOTE,
    aggregate_packed,
    aggregate_signs,
    apply,
    apply_encoded,
    build,
    compile_source,
    default,
    delta_planes,
    encode_delta,
    global_lion_step,
    step,
    step_mt,
    worker_step,
    worker_step_pw,
    words_for,
)

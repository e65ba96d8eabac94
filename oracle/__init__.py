"""fp64 CPU oracle of the TIDE router hot path (test infrastructure only).

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import
this package; the product library neither imports nor links it.
"""
from .tide_oracle import (  # noqa: F401
    DTYPE_CODES,
    batch_compact,
    batch_exit,
    build,
    cosine_labels,
    exit_from_fire,
    exit_project,
    round_to_storage,
    fires,
    max_threads,
    rmsnorm,
    router_eval,
    select_exit,
    set_threads,
    sigmoid,
    silu,
    widen,
)

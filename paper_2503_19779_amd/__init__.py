"""MI355X-native replay of a captured kernel chain with three input-refresh modes
(copy into placeholders, pointer-table indirection, per-segment selection).

Thin ctypes binding over libpygraph_hip.so; every step of the path runs in the HIP library.
"""
from .binding import (  # noqa: F401
    Chain,
    PgError,
    lib,
    select,
    eager_static,
    STATIC_SCRATCH_BYTES,
    version,
    EAGER,
    GRAPH_COPY,
    GRAPH_INDIRECT,
    SELECTED,
    GRAPH_UPDATE,
    TABLE_KERNARG,
    TABLE_MEMCPY,
    TABLE_GRAPH_MEMCPY,
    TABLE_HOST,
    COPY_KERNEL,
    COPY_MEMCPY,
)

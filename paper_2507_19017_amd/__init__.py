"""MI355X-native weight resharding (allgather-swap hot path): Python binding of libreshard.so."""

from .binding import (  # noqa: F401
    Plan,
    ReshardError,
    copy_baseline,
    read_baseline,
    write_baseline,
    get_tuning,
    last_error,
    redundant_memory_bytes,
    lib,
    set_host_limit,
    set_tuning,
    version,
)

"""FlashFPS-style farthest point sampling for MI355X (gfx950).

`binding` holds the Python front end of the C-ABI library (libflashfps.so,
built from csrc/ by build.py); `inputs` holds the seeded synthetic clouds used
by tests and benchmark."""
from .binding import (  # noqa: F401
    FFPS_FLAG_CP, FFPS_FLAG_IP, FFPS_FLAG_PERM, FFPS_MODE_CACHED, FFPS_MODE_CHAIN, FFPS_VARIANT_AUTO,
    FFPS_VARIANT_GRID, FFPS_VARIANT_STREAM, FFPS_VARIANT_WG, FlashFPSError, ffps_cached_stages,
    ffps_alu_probe, ffps_barrier_probe, ffps_describe_plan, ffps_exact, ffps_exact_noalloc, ffps_gather_rows, ffps_last_rounds, ffps_last_status, ffps_prune, ffps_prune_sizes, ffps_strerror, ffps_version,
    ffps_workspace_bytes, make_workspace,
)

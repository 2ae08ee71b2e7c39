"""MI355X-native hot path of the DHO2 / FOSI hybrid-order optimiser.

The arithmetic lives in libfosi_hip.so (hand-written HIP for gfx950, built by
`python -m paper_2505_00982_amd.build`); this package is a thin ctypes binding
with the same names as the C functions declared in include/fosi.h.
"""
from .binding import (  # noqa: F401
    FosiError,
    Context,
    Hvp,
    ColMajor,
    StepParams,
    fosi_lanczos,
    fosi_lanczos_begin,
    fosi_lanczos_end,
    fosi_lanczos_row_sharded,
    fosi_lanczos_steps,
    fosi_lanczos_second_passes,
    REORTH_SINGLE,
    REORTH_TWICE,
    REORTH_LOCAL_FULL,
    REORTH_SELECTIVE,
    GRAPH_OFF,
    GRAPH_ON,
    fosi_ritz,
    fosi_step,
    fosi_step_noalloc,
    fosi_step_adamw,
    AdamwParams,
    fosi_admm_begin,
    fosi_admm_end,
    fosi_traffic_model,
    fosi_tridiag_eigh,
    library_path,
    load_library,
    PROF,
    STATUS,
)

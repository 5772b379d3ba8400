"""MI355X (gfx950) implementation of AdaComp's data-parallel hot path.

Thin ctypes binding over libadacomp.so (C ABI in include/adacomp.h).  All
computation happens in the library's HIP kernels; this package only marshals
arguments.  PyTorch is used to own device memory and streams.
"""
from .binding import (  # noqa: F401
    AdaCompError,
    Update,
    Layers,
    Queue,
    State,
    adacomp_count,
    adacomp_select_workspace,
    adacomp_select,
    adacomp_select_noalloc,
    SELECT_NOALLOC_SCRATCH_BYTES,
    adacomp_apply_workspace,
    adacomp_apply,
    adacomp_apply_global_staleness,
    adacomp_update_validate,
    adacomp_wire_bound,
    adacomp_wire_workspace,
    adacomp_wire_pack,
    adacomp_wire_unpack,
    adacomp_strerror,
    adacomp_kernel_name,
    adacomp_profile_start,
    adacomp_profile_stop,
    library_path,
    load_library,
)

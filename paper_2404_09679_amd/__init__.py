"""MI355X (gfx950) library for one BSP Parameter-Server training iteration of a
ranking model: a thin ctypes binding over libantdt_hip.so (see include/antdt.h).

Every step of the iteration runs in the library's HIP kernels; this package only
marshals arguments.  There is no CPU fallback: importing `binding` raises if the
shared library has not been built (python paper_2404_09679_amd/build.py).
"""
from .binding import (  # noqa: F401
    AntdtError,
    Context,
    ShardQueue,
    simulate_bsp,
    Model,
    dense_aggregate_adam,
    expand_accumulation,
    fill_tables,
    kernel_names,
    lib,
    model_from_config,
    plan_accumulation,
    stream_copy,
)

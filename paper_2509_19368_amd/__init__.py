"""MI355X-native hot path of pipeline-parallel early-exit self-speculative decoding.

The work is done by hand-written HIP kernels in libppsd.so behind the C ABI of
include/ppsd.h; this package is the thin ctypes binding over it.  There is no
CPU fallback: importing the binding without the built library raises.
"""
from .binding import (  # noqa: F401
    ENGINE_PERSISTENT, ENGINE_STREAMS, MODE_EESD, MODE_OVERLAP, MODE_PIPELINE, MODE_SERIAL, MODE_VANILLA, KERNEL_KINDS, PpsdError, Session,
    hbm_read_probe, library_path, load_library, ppsd_workspace_bytes,
)

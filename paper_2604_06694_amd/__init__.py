"""MI355X (gfx950) implementation of AudioKV's prefill-time KV-cache eviction path.

The work is done by hand-written HIP kernels behind the C ABI declared in
include/audiokv.h (libaudiokv.so, built by paper_2604_06694_amd.build). This
package is only the ctypes binding: argument marshalling, with torch used for
device memory and streams. There is no CPU fallback: importing `binding`
without the built library raises.
"""
from .binding import (  # noqa: F401
    AudioKVError,
    Params,
    allocate,
    compact,
    evict,
    lib_path,
    n_keep,
    score,
    select,
    smooth,
    total_kept,
    version,
    workspace_bytes,
)

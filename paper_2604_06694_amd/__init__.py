"""MI355X (gfx950) implementation of AudioKV's prefill-time KV-cache eviction path.

The work is done by hand-written HIP kernels behind the C ABI declared in
include/audiokv.h (libaudiokv.so, built by `python -m paper_2604_06694_amd.build`).
This package is only the ctypes binding: argument marshalling, with torch used
for device memory and streams. There is no CPU fallback: the first use of any
binding name without the built library raises ImportError.

The binding is loaded on first attribute access so that the build module can be
run before the library exists.
"""
import importlib

_BINDING_NAMES = (
    "AudioKVError", "Params", "allocate", "compact", "decode_attend", "decode_workspace_bytes", "evict", "evict_noalloc", "lib_path", "n_keep", "profile_enable",
    "profile_read", "score", "select", "smooth", "smooth_cutoffs", "total_kept", "version", "workspace_bytes",
    "POOL_AVG", "POOL_MAX", "LAYOUT_HEAD_MAJOR", "LAYOUT_TOKEN_MAJOR", "SCOPE_ITEM", "SCOPE_GLOBAL",
    "CUTOFF_FRACTION", "CUTOFF_ENERGY", "CUTOFF_ENERGY_NO_DC",
    "PROFILE_STAGES", "NOALLOC_SCRATCH_BYTES",
)


def __getattr__(name):
    if name == "binding" or name in _BINDING_NAMES:
        b = importlib.import_module(".binding", __name__)
        value = b if name == "binding" else getattr(b, name)
        globals()[name] = value          # later lookups find it without coming through here
        return value
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")

"""CPU oracle for the AudioKV eviction path (test infrastructure only; see audiokv_oracle)."""
from . import audiokv_oracle  # noqa: F401

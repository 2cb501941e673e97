"""fp64 CPU oracle of the SamKV hot path (test infrastructure; never imported by the product path)."""
from . import samkv_oracle  # noqa: F401

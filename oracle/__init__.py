"""CPU oracle (test infrastructure only; never imported by the product path)."""
from . import sfmp_oracle  # noqa: F401

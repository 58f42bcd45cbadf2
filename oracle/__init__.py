"""CPU oracle package (test infrastructure only; never imported by the product path)."""
from . import psd_oracle  # noqa: F401

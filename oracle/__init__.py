"""CPU oracle package (test infrastructure only; see aug_oracle.py)."""
from . import aug_oracle  # noqa: F401

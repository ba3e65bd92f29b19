"""CPU oracle (test infrastructure only; the product path never imports this)."""
from . import confspec_oracle  # noqa: F401

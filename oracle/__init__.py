"""Plain CPU oracle of the HTTM global-attention layer.  Test infrastructure only:
imported by tests/, the smoke check and the benchmark's CPU-baseline leg, never by
the product package."""
from . import httm_oracle  # noqa: F401

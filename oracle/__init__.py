"""CPU oracle of the LGC compression path.  Test infrastructure only: see
lgc_oracle.c.  The product package never imports this."""
from . import lgc_oracle  # noqa: F401

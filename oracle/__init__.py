"""CPU oracle (test infrastructure only; never imported by the product path)."""
from .binding import (build, svdvals, bdsvals, bidiagonalize, householder,  # noqa: F401
                      num_threads)

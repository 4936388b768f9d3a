"""fp64 CPU oracle of the gated subspace linear layer (test infrastructure, not product code)."""
from .gsi_oracle import *  # noqa: F401,F403

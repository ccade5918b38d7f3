"""fp64 CPU oracle of the ZeCO GLA hot path.  Test infrastructure only (see gla_oracle.c)."""

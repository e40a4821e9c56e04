"""CPU oracle of the DGC hot path: test infrastructure only (see dgc_oracle)."""

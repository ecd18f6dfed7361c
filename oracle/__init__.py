"""CPU oracle of the IceCache hot path: test infrastructure only (see ice_oracle.c)."""

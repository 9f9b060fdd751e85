"""CPU oracle of the CO3 codec: test infrastructure only (see co3_oracle.c)."""

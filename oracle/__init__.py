"""CPU oracle of the SLIDE training step (test infrastructure; see slide_oracle.c)."""

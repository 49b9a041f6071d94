"""CPU oracle of the training step — test infrastructure only (see kge_oracle.c)."""

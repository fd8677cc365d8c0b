"""CPU oracle of the DHQ forward path (test infrastructure; see dhq_oracle.c)."""

"""CPU oracle of the ranking hot path -- test infrastructure only (see otf_oracle.c)."""

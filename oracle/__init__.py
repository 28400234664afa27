"""CPU oracle of the LP hot path -- test infrastructure only (see lp_oracle.c)."""

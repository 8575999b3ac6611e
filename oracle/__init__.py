"""CPU oracle for the EF21 hot path -- test infrastructure only (see ef21_oracle.c)."""

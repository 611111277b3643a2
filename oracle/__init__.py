"""CPU oracle package: test infrastructure only (see conv1d_oracle.c)."""

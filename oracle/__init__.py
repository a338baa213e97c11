"""Test infrastructure: plain CPU oracle of the simulated network (see gnr_oracle.c)."""

"""CPU float64 oracle: test infrastructure only (see fb_oracle.py)."""

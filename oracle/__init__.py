"""CPU oracle (test infrastructure only; see cachefocus_oracle.py)."""

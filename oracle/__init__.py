"""CPU oracle (test infrastructure only; see gtopk_oracle.py)."""

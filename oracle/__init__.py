"""CPU oracle (test infrastructure only; see sar_oracle.py)."""

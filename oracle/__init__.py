"""CPU oracle (test infrastructure only; see ee_oracle.py)."""

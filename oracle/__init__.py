"""CPU oracle (test infrastructure only; see cafeq_oracle.py)."""

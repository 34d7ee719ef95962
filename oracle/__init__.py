"""CPU oracle package: test infrastructure only (see cq_oracle.py)."""

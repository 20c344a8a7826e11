"""CPU oracle package (test infrastructure; see laserkv_oracle.py)."""

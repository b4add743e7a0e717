"""CPU oracle package (test infrastructure; see moqe_oracle.py)."""

"""fp64 CPU oracle (test infrastructure only; see sig_oracle.py)."""

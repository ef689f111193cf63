"""CPU oracle (test infrastructure only; see prefill_oracle.py)."""

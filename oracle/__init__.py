"""CPU oracle (test infrastructure).  See prefill_oracle.py."""

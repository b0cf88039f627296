"""fp64 CPU oracle (test infrastructure only; see burst_oracle.py)."""

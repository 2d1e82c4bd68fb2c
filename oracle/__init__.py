"""Float64 CPU checker (test infrastructure only; see aero_oracle.py)."""

"""Float64 CPU oracle (test infrastructure only; see leanquant_oracle.py)."""

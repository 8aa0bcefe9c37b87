"""Float64 CPU oracle (test infrastructure only; see demo_oracle.py)."""

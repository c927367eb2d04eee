"""CPU fp64 oracle for LoMA attention: test infrastructure only (see loma_oracle.py)."""

"""CPU oracle (test infrastructure). See chorus_oracle.py."""

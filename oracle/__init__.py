"""CPU oracle (test infrastructure): see slim_oracle.py."""

"""CPU oracle (test infrastructure): see lens_oracle.py."""

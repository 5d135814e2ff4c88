"""CPU oracle (test infrastructure only): see cat_oracle.py."""

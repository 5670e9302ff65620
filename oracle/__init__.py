"""CPU oracle (test infrastructure). See approxifer_oracle.py."""

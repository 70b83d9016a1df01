"""CPU oracle (test infrastructure). See mate_oracle.py."""

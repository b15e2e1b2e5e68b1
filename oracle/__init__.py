"""CPU oracle (test infrastructure).  See hla_oracle.py."""

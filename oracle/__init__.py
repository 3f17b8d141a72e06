"""CPU oracle (test infrastructure).  See locret_oracle.py."""

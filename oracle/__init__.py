"""CPU oracle (test infrastructure only).  See lp_oracle.py."""

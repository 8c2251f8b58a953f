"""CPU oracle (test infrastructure).  See pf_oracle.c and pf_oracle.py."""

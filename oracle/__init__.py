"""CPU oracle (test infrastructure only): see qp_oracle.c and qp_oracle.py."""

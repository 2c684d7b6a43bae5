"""CPU oracle (test infrastructure only): see oracle/bnn_oracle.c and oracle/oracle.py."""

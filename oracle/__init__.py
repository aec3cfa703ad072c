"""CPU oracle (test infrastructure only). See oracle/conv_oracle.c and oracle/oracle.py."""

"""CPU oracle (test infrastructure only). See oracle/lrbi_oracle.py."""

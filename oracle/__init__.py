"""CPU checker for the PeRQ activation path.  Test infrastructure only -- see perq_oracle.py."""

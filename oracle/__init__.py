"""CPU oracle (test infrastructure).  See oracle/backprop.py."""

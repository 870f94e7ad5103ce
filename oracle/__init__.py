"""TEST INFRASTRUCTURE: the fp64 CPU oracle (see rfast_oracle.py).  Not part of the product path."""

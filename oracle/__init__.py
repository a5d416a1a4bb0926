"""Float64 CPU oracle for CGBN.  Test infrastructure: see cgbn_oracle.py."""

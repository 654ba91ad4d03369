"""fp64 CPU oracle for Selective Head Attention.  Test infrastructure only; see polar_oracle.c."""

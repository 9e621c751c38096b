"""fp64 CPU oracle for packed variable-length attention.  Test infrastructure only."""

"""fp64 CPU oracle for MLA decode attention.  Test infrastructure only."""

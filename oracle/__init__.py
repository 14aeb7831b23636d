"""fp64 CPU oracle for the TWA projected step.  Test infrastructure only -- never imported by the product."""

"""fp64 CPU oracle for the DVP row path (test infrastructure, not product code)."""

"""fp64 CPU oracle for the K-FAC work items: test infrastructure, not product code."""

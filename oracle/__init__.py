"""fp64 CPU oracle for the linear cross-entropy path: test infrastructure, not product code."""

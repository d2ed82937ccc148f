"""CPU oracle for the BRACE aggregation path -- test infrastructure, never used by the product path."""

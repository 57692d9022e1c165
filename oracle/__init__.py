"""CPU oracle for the TBE operator: test infrastructure only, never imported by the product path."""

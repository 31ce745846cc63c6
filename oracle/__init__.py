"""CPU oracle for GQLA decode attention: test infrastructure, never on the product path."""

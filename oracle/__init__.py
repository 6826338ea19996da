"""CPU oracle for the GANQ layer solver: test infrastructure, never on the product path."""

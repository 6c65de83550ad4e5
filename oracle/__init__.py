"""CPU oracle for the Ecco codec -- test infrastructure only; never imported by the product path."""

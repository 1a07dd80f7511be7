"""CPU oracle for the QSDP codec: test infrastructure, never part of the product path."""

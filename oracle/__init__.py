"""CPU oracle of the MEFT sparse-adapter layer: test infrastructure, never on the product path."""

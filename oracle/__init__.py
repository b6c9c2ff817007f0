"""CPU oracle of the DSA forward path: test infrastructure only, never a product path."""

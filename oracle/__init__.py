"""fp64 CPU oracle of the merge step: test infrastructure, never on the product path."""

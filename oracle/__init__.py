"""fp64 CPU oracle of the compression pass: test infrastructure, never on the product path."""

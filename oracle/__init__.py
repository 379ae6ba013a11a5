"""CPU fp64 oracle of the ISOPO layer step: test infrastructure, never on the product path."""

"""CPU oracle of the reduction path: test infrastructure, never a product dependency."""

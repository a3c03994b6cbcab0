"""CPU oracle of the sparse-FFN hot path: test infrastructure, never imported by the product path."""

"""CPU oracle of the attention-carving hot path: test infrastructure, never imported by the product."""

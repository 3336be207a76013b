"""CPU oracle of the IST hot path: test infrastructure, never used by the product."""

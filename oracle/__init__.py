"""CPU oracle of the PAAC hot path: test infrastructure, never imported by the product path."""

"""CPU oracle of the EpiCache eviction step: test infrastructure, never imported by the product package."""

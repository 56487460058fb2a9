"""CPU oracle of the Bolt hot path: test infrastructure, never imported by the product package."""

"""CPU oracle of the LRSA hot path: test infrastructure, never imported by the product package."""

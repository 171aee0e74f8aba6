"""CPU oracle of the CalibQuant hot path: test infrastructure, never imported by the product."""

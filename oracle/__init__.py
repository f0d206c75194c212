"""CPU oracle of the Kascade hot path: test infrastructure, never imported by the product."""

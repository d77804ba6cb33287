"""CPU oracle of the LRQK decode step — test infrastructure, not part of the product."""

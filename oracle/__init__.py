"""Float64 CPU oracle of the ESA step: test infrastructure, never part of the product path."""

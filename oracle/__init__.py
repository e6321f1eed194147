"""CPU oracle of the GWQ linear-layer path: test infrastructure, never part of the product path."""

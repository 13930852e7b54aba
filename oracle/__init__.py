"""fp64 CPU oracle of the Partial FC step: test infrastructure, never imported by the product."""

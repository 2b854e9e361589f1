"""CPU oracle of the RPTQ hot path: test infrastructure, never a product path."""

"""CPU oracle of the Medusa verification step: test infrastructure, not product code."""

"""CPU oracle of the PPLL local-block step: test infrastructure, not product code."""

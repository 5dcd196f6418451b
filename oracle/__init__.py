"""CPU oracle of the SAT partition step: test infrastructure, not product code."""

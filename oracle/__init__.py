"""CPU oracle for the structured-OBS pruner: test infrastructure, not product code."""

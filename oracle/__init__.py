"""CPU oracle (test infrastructure only): untiled forward/backward and the integer tile maps."""

"""CPU oracle of the rehearsal-buffer path: test infrastructure, never part of the product path."""

"""CPU oracle of the SLICER IF codec: test infrastructure, never a product path."""

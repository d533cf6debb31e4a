"""CPU oracle of the MXInt format and product -- test infrastructure, not part of the library."""

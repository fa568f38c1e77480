"""CPU oracle of the tropical convolution family: test infrastructure, never the product path."""

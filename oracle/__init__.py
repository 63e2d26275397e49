"""CPU oracle for the SVDQuant linear layer: test infrastructure, never imported by the product path."""

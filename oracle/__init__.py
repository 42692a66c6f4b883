"""CPU oracle for the 3D convolutional layer -- test infrastructure, never part of the product path."""

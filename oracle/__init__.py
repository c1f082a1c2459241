"""CPU oracle of the STaMP linear layer.  Test infrastructure: not imported by the product path."""

"""CPU oracle for the block-structured-pruned linear layer.  Test infrastructure only:
nothing in the product package may import this."""

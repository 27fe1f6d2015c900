"""CPU oracle of the 8-bit NMT decoding hot path.  Test infrastructure only:
nothing in the product package may import this."""

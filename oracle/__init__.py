"""CPU oracle of the pattern-sparse convolution path. Test infrastructure: never imported by the product."""

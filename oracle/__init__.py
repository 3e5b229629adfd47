"""CPU oracle of the MoFQ quantize-and-score path: test infrastructure only."""

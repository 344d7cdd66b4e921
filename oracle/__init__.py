"""CPU oracle of the checkpoint-compressor hot path: test infrastructure only."""

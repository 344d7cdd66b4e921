"""MI355X-native hot path of the checkpoint compressor (search, quantize, delta)."""

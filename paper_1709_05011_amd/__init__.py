"""MI355X-native convolution + LARS training hot path (see ``larsconv`` for the binding)."""

"""MI355X-native structured-OBS pruning hot path (ZipLM, Section 3.1 / Algorithm 1)."""

"""MI355X-native batched evaluation of candidate operator schedules (arxiv 2503.09357 hot path)."""

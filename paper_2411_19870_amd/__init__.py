"""MI355X-native DeMo per-step compression path (encode / decode / step)."""

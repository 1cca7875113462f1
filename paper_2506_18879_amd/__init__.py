"""MI355X-native decode attention over a CommVQ-compressed KV cache (libcommvq binding)."""

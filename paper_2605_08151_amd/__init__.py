"""MI355X-native target-side verification step (verify attention, LM head, acceptance, KV commit)."""

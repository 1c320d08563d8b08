"""MI355X-native chunked-prefill attention over a paged KV cache (TetriInfer prefill hot path)."""

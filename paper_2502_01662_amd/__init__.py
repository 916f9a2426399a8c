"""MI355X-native batched verification step of Collaborative decoding via Speculation."""

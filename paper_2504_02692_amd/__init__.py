"""MI355X-native GPTAQ per-layer solve (accumulate -> prepare -> quantize)."""

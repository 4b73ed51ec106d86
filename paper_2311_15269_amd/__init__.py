"""MI355X-native batched evaluation of Tessel repetend candidates (hot path only)."""

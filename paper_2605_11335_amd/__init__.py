"""MI355X-native block path for layerwise-offloaded DiT inference (HIP library + thin binding)."""

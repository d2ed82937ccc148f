"""MI355X-native BRACE robust chunk aggregation (Byzantine-robust ring-all-reduce)."""

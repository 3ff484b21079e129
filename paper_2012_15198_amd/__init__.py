"""MI355X-native segment-wise gossip parameter mixing (Crossover-SGD hot path)."""

"""MI355X-native linked-operator-chain CNN inference (hot path of arxiv 2302.00282)."""

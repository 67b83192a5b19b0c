"""MI355X-native LQ decomposition (low-rank plus NF-quantized) hot path."""

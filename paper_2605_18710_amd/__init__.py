"""MI355X-native hot path of temporal-spatial module multiplexing (one GPU)."""

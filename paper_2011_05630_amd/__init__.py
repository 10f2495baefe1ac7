"""MI355X-native fused-layer CNN execution (DLFusion's hot path): C-ABI library + thin binding."""

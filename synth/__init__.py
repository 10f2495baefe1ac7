"""Seeded synthetic workloads (layer shapes and tensors); holds none of the method's arithmetic."""

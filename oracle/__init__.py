"""CPU oracle: test infrastructure only. Nothing in the GPU library imports this package."""

"""CPU checker (test infrastructure only; never imported by the GPU library)."""

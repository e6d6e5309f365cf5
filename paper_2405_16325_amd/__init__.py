"""MI355X-native double-pruned 2:4 sparse linear layer (SLoPe hot path).

``binding`` wraps the C-ABI library built from ``csrc/``; ``inputs`` draws the
seeded synthetic operands.  There is no CPU fallback: every call runs in the HIP
kernels, and loading fails loudly if the library has not been built.
"""

"""MI355X-native tropical convolution (max-plus / min-plus / compound / parallel), forward and backward.

The compute path is the C-ABI library built from ``csrc/`` (see ``include/tconv.h``);
``binding`` marshals arguments to it and ``inputs`` draws seeded synthetic tensors.
Nothing here falls back to a CPU implementation: a missing library is an error.
"""
__all__ = ["binding", "inputs"]

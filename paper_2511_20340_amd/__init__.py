"""MI355X-native (gfx950) draft / verify / accept step of SpecFormer-style speculative decoding.

The product is the C-ABI library libspecformer.so (include/specformer.h); this package is its
thin Python binding: `binding` mirrors the C entry points one to one, `engine` owns the device
buffers (PyTorch tensors) and passes their pointers.  Nothing here computes any step of the path.
"""
__all__ = ["binding", "engine", "metrics"]

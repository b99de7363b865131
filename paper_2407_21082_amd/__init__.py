"""MI355X-native early-exit head evaluation and DSSD greedy verification
(arXiv 2407.21082).  The compute lives in libeh.so (hand-written HIP for
gfx950, C ABI in include/eh.h); ``binding`` marshals torch tensors into it."""
__all__ = ["binding", "build"]

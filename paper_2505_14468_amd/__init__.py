"""MI355X-native multi-LoRA batched linear layer: thin Python binding over the
C-ABI library ``liblora_mi355x.so`` (hand-written HIP kernels for gfx950).

Importing the package loads nothing; ``paper_2505_14468_amd.binding`` loads the
shared library and raises if it has not been built (there is no fallback path).
"""
__all__ = ["binding", "runtime", "build"]

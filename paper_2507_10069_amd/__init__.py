"""MI355X-native prefix-cached paged prefill attention (KV scatter, causal GQA prefill over a
paged pool with a cached multimodal prefix, and the mask-free cross-attention variant).

The compute lives in a C-ABI HIP library (``include/emm.h``); :mod:`.binding` marshals
arguments to it.  Importing this package does not load the library; the first call through
:mod:`.binding` does, and raises if it has not been built."""

__all__ = ["workloads", "binding", "build"]

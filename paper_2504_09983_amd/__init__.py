"""MI355X-native sharded optimizer step (fused Adam(W), bf16 cast, unshard, offload).

``paper_2504_09983_amd.zc`` is the thin binding over the C-ABI library
(``include/zc.h``); ``paper_2504_09983_amd.synth`` draws seeded synthetic
inputs.  Importing the package loads nothing; the shared library is loaded on
first use of ``zc`` and its absence is an error, never a fallback.
"""
__all__ = ["zc", "synth"]

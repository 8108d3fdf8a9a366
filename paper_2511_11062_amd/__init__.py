"""MI355X-native LiteAttention hot path: a C-ABI HIP library (csrc/) and its thin Python binding.

``inputs`` (synthetic data) imports nothing native; ``lite_attn`` loads the built shared library and
raises if it is missing -- there is no CPU fallback.
"""

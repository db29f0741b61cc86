"""s3kv: prediction-sized ragged KV cache + decode-step attention for MI355X (gfx950).

``binding`` is the thin ctypes layer over ``libs3kv.so`` (same names as the C ABI);
``workloads`` draws the seeded synthetic inputs; ``build`` compiles the library.
Nothing is loaded at import time; ``binding.lib()`` fails loudly when the HIP
library has not been built.
"""

"""MI355X-native adaptive mixed-precision KV-cache decoding (features, controller, append, decode attention).

``binding`` wraps the C ABI of ``libkvq.so`` (hand-written HIP for gfx950); ``build`` compiles the library.  Nothing here computes any step of the method in
Python, and there is no CPU fallback.
"""

__all__ = ["binding", "build"]

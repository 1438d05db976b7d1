"""MI355X-native batched hybrid KV-cache restoration (CacheFlow's hot path).

Thin ctypes binding over libcacheflow.so; every step of the path runs in the
library's HIP kernels and host C++.  There is no CPU fallback: touching any
binding name without the built library raises ImportError.  (The binding is
loaded on first use so that `python -m paper_2604_25080_amd.build` can run
before the library exists.)"""
import importlib

_binding = None


def __getattr__(name):
    global _binding
    if name.startswith("__"):
        raise AttributeError(name)
    if _binding is None:
        _binding = importlib.import_module(".binding", __name__)
    if name == "binding":
        return _binding
    return getattr(_binding, name)

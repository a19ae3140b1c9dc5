"""MI355X-native verification hot path of Lookahead Reasoning (arXiv 2506.19830).

``la_verify_attention`` and ``la_spec_accept`` are thin ctypes bindings of the
C-ABI library built from ``csrc/``; every step of the path runs in its HIP
kernels.  Importing the package does not load the library; the first call does
and raises if it has not been built.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    if name in ("la_verify_attention", "la_spec_accept", "la_verify_attention_workspace", "la_spec_accept_workspace"):
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)

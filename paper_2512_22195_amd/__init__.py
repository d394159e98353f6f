"""MatKV inference hot path on MI355X: Python face of libmatkv.so.

``build.build()`` compiles the library; everything else lives in ``binding`` and is
loaded on first use.  There is no CPU fallback: touching any entry point without a
built library raises ImportError.
"""
from .build import LIB_PATH, build

__all__ = ["build", "LIB_PATH", "binding"]


def __getattr__(name):
    if name == "binding" or not name.startswith("_"):
        import importlib
        b = importlib.import_module(".binding", __name__)
        if name == "binding":
            return b
        try:
            return getattr(b, name)
        except AttributeError:
            raise AttributeError(f"module {__name__!r} has no attribute {name!r}") from None
    raise AttributeError(name)

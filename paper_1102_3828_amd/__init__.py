"""IVFADC+R search (arXiv 1102.3828) on MI355X: ctypes binding over the HIP library.

The binding is loaded on first use, so that `paper_1102_3828_amd.build` can be imported (and run)
before the library exists.  Using the package without a built library raises ImportError."""
import importlib

_BINDING_NAMES = ("Index", "IvfrError", "EXPORTED", "LIB_PATH", "lib", "memory_required")


def __getattr__(name):
    if name == "binding" or name in _BINDING_NAMES:
        binding = importlib.import_module(".binding", __name__)
        return binding if name == "binding" else getattr(binding, name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")

"""IVFADC+R search (arXiv 1102.3828) on MI355X: ctypes binding over the HIP library."""
from .binding import Index, IvfrError, EXPORTED, LIB_PATH, lib  # noqa: F401

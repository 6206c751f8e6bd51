"""DEER draft-verify step on MI355X: thin Python binding over libdeer's C ABI."""
from .binding import DeerEngine, DeerError, load_library, LIB_PATH  # noqa: F401

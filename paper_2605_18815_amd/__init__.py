"""MI355X-native Virtual Parameter Space state-transition engine (HIP library + ctypes binding)."""
from .binding import Library, VpsError, BOX_DTYPE, PIECE_DTYPE, NO_POS  # noqa: F401

_default = None


def load():
    """The process-wide library instance (loads paper_2605_18815_amd/libvps.so)."""
    global _default
    if _default is None:
        _default = Library()
    return _default

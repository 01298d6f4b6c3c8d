"""MI355X-native AdaCons gradient aggregation: HIP kernels behind a C ABI, ctypes binding."""
from .binding import *  # noqa: F401,F403
from .binding import AdaCons, AdaConsError, AdaConsLayers, EXPORTS, library_path

__all__ = [n for n in dir() if n.startswith(("adacons_", "ADACONS_"))] + ["AdaCons", "AdaConsError", "AdaConsLayers", "EXPORTS", "library_path"]

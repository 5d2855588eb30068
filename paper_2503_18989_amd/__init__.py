"""MI355X-native middle-submodel forward of HAT (arXiv 2503.18989).

Thin ctypes binding over libhatmid.so (hand-written HIP for gfx950).  The
binding only marshals arguments; every step of the path runs in the library's
kernels.  There is no CPU fallback: without the built library, import of
`paper_2503_18989_amd.binding` raises.
"""
from .binding import (HatMid, HatPlanner, HatSched, HatError, Segment, CHUNK, VERIFY, lib_path, load_library,  # noqa: F401
                      KERNEL_NAMES, DUMP_IDS, EXPORTED_SYMBOLS)

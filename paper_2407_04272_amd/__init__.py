"""MI355X-native error-bounded compressor for DLRM embedding all-to-all payloads (arXiv 2407.04272).

``csrc/`` holds the HIP kernels and the C ABI (``include/dlc.h``); ``binding`` is the ctypes layer
with the same names; ``build`` compiles ``libdlc.so`` in-tree for gfx950.
"""
from . import binding  # noqa: F401
from .binding import (Context, ControllerParams, DlcError, TableStats, dlc_compress_bound, dlc_strerror,  # noqa: F401
                      dlc_workspace_bytes, make_config)

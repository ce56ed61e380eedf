"""MI355X-native shape-generic fusion kernels behind a C ABI (see include/disc.h).

Python here is argument marshalling only: every step of the path (constraint closure,
fusion decision, code generation, the one device compile, shape calculation, version
selection, launch) runs inside libdisc.so and its gfx950 kernels.
"""
from .binding import (BoundCall, Context, DiscError, PatternHandle, lib_path, load_library,  # noqa: F401
                      OPCODE_IDS, DTYPE_IDS, VARIANTS, STATUS)

"""MI355X (gfx950) draft-tree verification: hand-written HIP kernels behind a C ABI.

`binding` mirrors the entry points of include/ded_verify.h; `build.build_library()` compiles the
shared library in-tree.  Nothing here falls back to a CPU path: without the library every call raises.
"""
from . import binding  # noqa: F401
from .binding import Verifier, Drafter, DedError  # noqa: F401

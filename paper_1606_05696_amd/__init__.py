"""StridedBatchedGemm and copy-free tensor contractions for AMD MI355X (gfx950).

The work is done by libsbgemm.so (hand-written HIP kernels behind a C ABI, see include/sbgemm.h);
`binding` exposes its entry points under the same names.  The library is loaded on first use and
there is no fallback path: calls raise if it has not been built.
"""
from .binding import *  # noqa: F401,F403
from .binding import SbError, sb_plan  # noqa: F401

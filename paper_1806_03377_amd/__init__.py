"""MI355X-native 1F1B weight-stashed pipeline-stage runtime (PipeDream, arXiv 1806.03377).

The work is done by libpd.so (HIP kernels + C ABI, see include/pd.h); this package is
its thin ctypes binding.  There is no CPU fallback: importing `binding` fails if the
library has not been built (`python -m paper_1806_03377_amd.build`).
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403

"""IntSGD compression hot path for MI355X: thin Python binding of the C-ABI HIP library.

Every arithmetic step runs in the library's kernels (csrc/); this package only
marshals arguments.  PyTorch is used for device memory and streams.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
from .placement import HBM_REGIONS, Arena  # noqa: F401

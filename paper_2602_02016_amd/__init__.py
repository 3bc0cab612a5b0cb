"""MI355X-native hot path of DASH's block-diagonal Shampoo step.

The product is the C-ABI library `libdash.so` (include/dash.h, sources under csrc/);
`binding` is a thin ctypes layer with the same call names that marshals device
pointers of torch tensors.  Importing this package does not load the library; the
first use of `binding.Dash` does, and fails loudly if it has not been built.
"""
from . import binding  # noqa: F401
from .binding import Dash, DashError, DashModel, chebyshev_fit, load_library, model_plan  # noqa: F401

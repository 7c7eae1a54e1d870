"""MI355X-native execution of fused tensor-operator groups of a shape-typed
graph: a C-ABI library (librelayhip.so, HIP kernels for gfx950 + host planner)
and its ctypes binding.  There is no CPU or eager fallback: without the built
library every entry point raises."""
from . import binding  # noqa: F401
from .binding import Context, Graph, Plan, RelayError, graph_from_spec, lib  # noqa: F401

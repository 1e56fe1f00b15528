"""MI355X-native normalized-adjacency propagation (LightGCN-style message passing).

`binding` mirrors the C ABI of libe2eg.so one to one (argument marshalling only);
`device` adds buffer allocation through torch so callers do not size workspaces by hand.
All arithmetic runs in the HIP kernels of libe2eg.so; there is no fallback path.
"""
from . import binding  # noqa: F401
from .binding import E2egError, load_library  # noqa: F401

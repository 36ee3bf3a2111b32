"""MI355X-native GNN aggregation library (GNNAdvisor's hot path) -- Python binding.

The compute lives in ``libgnn_mi355x.so`` (hand-written HIP for gfx950 behind the C ABI of
``include/gnn.h``).  This package only marshals arguments: torch is used for device memory
and streams, numpy for host arrays.  There is no CPU fallback: if the library is missing,
importing :mod:`paper_2006_06608_amd.binding` raises.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401

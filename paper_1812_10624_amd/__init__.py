"""MI355X-native library for one GPU's share of a layer-separated training iteration.

`api` binds the C ABI of libstanza.so one to one; `netrun` sequences those calls for a CONV worker,
the FC worker and the gradient aggregation.  The HIP library is the only compute path.
"""
from . import api  # noqa: F401

__all__ = ["api"]

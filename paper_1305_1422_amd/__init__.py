"""Batch self-organizing-map training on one AMD MI355X: binding of the HIP library libsom.

``capi`` mirrors ``include/som.h`` name for name; ``Som`` is a convenience wrapper holding
torch tensors.  The library must have been built (``python -m paper_1305_1422_amd.build``).
"""
from . import capi  # noqa: F401

__all__ = ["capi", "Som"]


def __getattr__(name):
    if name == "Som":
        from .som import Som
        return Som
    raise AttributeError(name)

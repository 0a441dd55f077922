"""MI355X-native batched truncated path-signature transform.

The compute path is the C-ABI library built from csrc/ (hand-written HIP for
gfx950); `signature` and friends in `binding` marshal arguments only.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)

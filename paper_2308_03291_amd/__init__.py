"""MI355X-native batched linear-chain CRF inference (log-partition, marginals, argmax).

The compute lives in ``csrc/`` (hand-written HIP for gfx950 behind a C ABI declared in
``include/lccrf.h``).  ``binding`` marshals torch device tensors to that ABI; ``workloads``
draws the seeded synthetic inputs.  Importing the package does not load the shared
library; the first call into ``binding`` does, and fails loudly when it is missing.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)

"""MI355X-native chunk-backed KV tensors, KV append and batched GQA decode attention
(the data-parallel hot path of the eLLM elastic memory framework, arXiv 2506.15155).

This package is a thin ctypes binding over libellm.so (hand-written HIP for gfx950). It only
marshals arguments; every step of the path runs in the library. Importing it without a built
library raises: there is no fallback path.
"""
from . import binding
from .binding import EllmError, ERR, LIB_PATH, lib  # noqa: F401

# every function of include/ellm.h under its own name, and the header's constants
for _name in dir(binding):
    if _name.startswith(("ellm_", "ELLM_")):
        globals()[_name] = getattr(binding, _name)
del _name

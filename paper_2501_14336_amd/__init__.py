"""Radix top-k selection for AMD Instinct MI355X (gfx950).

``rtopk_select`` & co. are thin bindings over the C-ABI library built from
``csrc/`` (see ``binding.py``); ``workloads`` holds the seeded input generators.
The library is loaded on first use, so importing the package needs no GPU.
"""
import importlib

from . import workloads  # noqa: F401

_BINDING_NAMES = (
    "rtopk_workspace_bytes", "rtopk_select", "rtopk_status_string", "rtopk_version", "topk", "read_trace",
    "build", "load", "RtopkTuning", "RtopkError", "RTOPK_F32", "RTOPK_F16", "RTOPK_BF16", "RTOPK_FLAG_SCALING",
)


def __getattr__(name):
    # bindings resolve lazily: `import paper_2501_14336_amd` must work where nothing is built yet
    if name in _BINDING_NAMES:
        return getattr(importlib.import_module(__name__ + ".binding"), name)
    raise AttributeError("module %r has no attribute %r" % (__name__, name))

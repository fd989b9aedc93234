"""Radix top-k selection for AMD Instinct MI355X (gfx950).

``rtopk_select`` & co. are thin bindings over the C-ABI library built from
``csrc/`` (see ``binding.py``); ``workloads`` holds the seeded input generators.
The library is loaded on first use, so importing the package needs no GPU.
"""
from . import workloads  # noqa: F401


def __getattr__(name):
    # bindings are resolved lazily: `import paper_2501_14336_amd` must work where nothing is built yet
    from . import binding
    try:
        return getattr(binding, name)
    except AttributeError:
        raise AttributeError("module %r has no attribute %r" % (__name__, name)) from None
